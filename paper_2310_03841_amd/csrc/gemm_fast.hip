// Fast path of the protected GEMM for gfx950: B stored N x K (both operands K-contiguous) and
// K a whole number (at least three) of 128-byte slabs.  Same mathematics, the same pass over
// A's slabs and the same epilogue as gemm_kernel; what differs is the data movement:
//   * global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4): no VGPR staging.  One
//     wave instruction fills 8 LDS rows of 128 bytes; the XOR swizzle of the LDS layout is
//     applied by choosing which global 16-byte chunk each lane fetches.
//   * 256 x 256 tiles, 4 waves of 128 x 128 (sixteen 32x32 MFMA blocks per wave), two LDS
//     buffers of 64 KB, one barrier per slab; 128 x 256 tiles fill the last, partial round.
//   * the loads of the next-but-one slab are issued one by one between the MFMAs of a slab's
//     last step, without branches.
//   * MFMAs take the B fragment first, so a lane owns a row of C (see gemm_epilogue.h).
//   * workgroup -> tile mapping keeps the workgroups that share an XCD (and its L2) on a
//     compact group of tiles.
// Rows of the tile beyond the problem are fetched from a valid row instead of being
// zero-filled: a row of A only influences the same row of C, which is discarded, and the pass
// over A's slabs ignores them.
#include <mutex>
#include <queue>
#include <vector>

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

    const int tid = tile_thread_index(), lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform by construction
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int M = g.M, N = g.N, K = g.K;

    const uint8_t *Ab = g.A + (long)bz * g.sA * ES;
    const uint8_t *Bb = g.B + (long)bz * g.sB * ES;

    // ---- global sources.  Load group p of this wave covers tile rows (4 p + wave) * 8 .. + 8;
    // lane l lands in LDS row + (l >> 3), slot (l & 7), and fetches the chunk for which
    // LDS slot = chunk ^ ((row >> 1) & 7).  (A 16-byte fragment read is served sixteen lanes at a
    // time from 64 banks: sixteen consecutive rows must fall on sixteen different 16-byte bank
    // groups.  Two consecutive 128-byte rows span all 64 banks, so the eight even rows need eight
    // different slots, and so do the eight odd rows; chunk ^ (row & 7) makes rows r and r + 8
    // collide, which the LDS bank-conflict counter showed as half of all LDS cycles.)  An address is a wave-uniform base (tile origin plus
    // the slab's offset along K) plus a per-lane 32-bit offset that never changes, so issuing a
    // load inside the main loop costs no vector arithmetic and no branch.  Rows of the tile past
    // the end of the matrix fetch the last valid row instead.
    const int lrow = lane >> 3;
    const int lchunk = (lane & 7) ^ (((wave & 1) << 2) + (lrow >> 1));
    const uint8_t *a_base = Ab + (long)m0 * g.lda * ES;
    const uint8_t *b_base = Bb + (long)n0 * g.ldb * ES;
    uint32_t a_off[GA], b_off[GB];
#pragma unroll
    for (int p = 0; p < GA; ++p) {
        int r = (4 * p + wave) * 8 + lrow;
        r = r < M - m0 ? r : M - m0 - 1;
        a_off[p] = (uint32_t)r * (uint32_t)(g.lda * ES) + lchunk * 16;
    }
#pragma unroll
    for (int p = 0; p < GB; ++p) {
        int r = (4 * p + wave) * 8 + lrow;
        r = r < N - n0 ? r : N - n0 - 1;
        b_off[p] = (uint32_t)r * (uint32_t)(g.ldb * ES) + lchunk * 16;
    }
    const int a_rows = M - m0;                        // rows of this tile inside A

    // The accumulators are never zero-filled: the first MFMA of every block takes a literal
    // zero as its addend.  Every block is always computed, also where the tile hangs over the
    // edge of the problem: a conditional MFMA would force the accumulators out of the AGPRs.
    accv_t acc[MI][NI];
    accv_t zerov;
#pragma unroll
    for (int i = 0; i < 16; ++i) zerov[i] = T::zero();

    auto issue_loads = [&](int s, int buf) __attribute__((always_inline)) {
        const uint8_t *ak = a_base + (long)s * SLAB_BYTES;
        const uint8_t *bk = b_base + (long)s * SLAB_BYTES;
        uint8_t *sA = smem + buf * BUF;
        uint8_t *sB = sA + BM * SLAB_BYTES;
#pragma unroll
        for (int p = 0; p < GA; ++p)
            __builtin_amdgcn_global_load_lds((gas_ptr)(ak + a_off[p]), (las_ptr)(sA + (4 * p + wave) * 8 * SLAB_BYTES), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < GB; ++p)
            __builtin_amdgcn_global_load_lds((gas_ptr)(bk + b_off[p]), (las_ptr)(sB + (4 * p + wave) * 8 * SLAB_BYTES), 16, 0, 0);
    };
    // ---- main loop, software-pipelined by hand.  A slab is four MFMA steps of 32 bytes of K.
    // The fragments of step t+1 are read from LDS while the MFMAs of step t run (two register
    // sets); the reads are issued in the first half of a step so that the second half covers
    // their latency.  The barrier sits between steps 2 and 3: by then every wave has read its
    // step-3 fragments, so nobody reads this slab's buffer any more and the loads of slab s+2
    // are issued into it at once, spread between the MFMAs of step 3, which also prefetches
    // step 0 of slab s+1.  The loop is peeled (first slab: literal-zero addend; last two slabs:
    // nothing left to load) so that no branch separates loads and MFMAs.
    i32x4 fa[2][MI], fb[2][NI];
    auto ldfr = [&](int buf, int s4, int set) __attribute__((always_inline)) {
        const uint8_t *sA = smem + buf * BUF;
        const uint8_t *sB = sA + BM * SLAB_BYTES;
        const int sw = ((2 * s4 + lh) ^ ((lane >> 1) & 7)) * 16;
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
    // Step 3 of a slab that still has loads to issue, in explicit program order: after every
    // MFMA (register set 1) one fragment read of the next slab's step 0 (into set 0) while
    // there are any, and this MFMA's share of the GA + GB direct-to-LDS loads of slab s + 2.
    // The scheduling fences keep that order; left alone, the compiler issues all loads in one
    // burst behind the barrier and the matrix pipe waits for them.
    auto step3_loads = [&](int s2, int buf) __attribute__((always_inline)) {
        constexpr int NMF = MI * NI, NLD = GA + GB;
        const uint8_t *ak = a_base + (long)s2 * SLAB_BYTES;
        const uint8_t *bk = b_base + (long)s2 * SLAB_BYTES;
        uint8_t *dA = smem + buf * BUF;
        uint8_t *dB = dA + BM * SLAB_BYTES;
        const uint8_t *sA = smem + (buf ^ 1) * BUF;
        const uint8_t *sB = sA + BM * SLAB_BYTES;
        const int sw = (lh ^ ((lane >> 1) & 7)) * 16;
        static_for<0, NMF>([&](auto j_c) {
            constexpr int j = decltype(j_c)::value;
            constexpr int mi = j / NI, ni = j % NI;
            acc[mi][ni] = T::mfma(fb[1][ni], fa[1][mi], acc[mi][ni]);
            if constexpr (j < MI)
                fa[0][j] = *reinterpret_cast<const i32x4 *>(sA + (wm * TM + j * 32 + l32) * SLAB_BYTES + sw);
            else if constexpr (j < MI + NI)
                fb[0][j - MI] = *reinterpret_cast<const i32x4 *>(sB + (wn * TN + (j - MI) * 32 + l32) * SLAB_BYTES + sw);
            constexpr int l0 = j * NLD / NMF, l1 = (j + 1) * NLD / NMF;
            static_for<l0, l1>([&](auto l_c) {
                constexpr int l = decltype(l_c)::value;
                if constexpr (l < GA)
                    __builtin_amdgcn_global_load_lds((gas_ptr)(ak + a_off[l]), (las_ptr)(dA + (4 * l + wave) * 8 * SLAB_BYTES), 16, 0, 0);
                else
                    __builtin_amdgcn_global_load_lds((gas_ptr)(bk + b_off[l - GA]), (las_ptr)(dB + (4 * (l - GA) + wave) * 8 * SLAB_BYTES), 16, 0, 0);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // Protected tiles reduce the slabs of A they own (slab s belongs to tile column s mod
    // tiles_n) while those are resident: see gemm_apass.h.
    constexpr int AUX_OFF = 2 * (256 + 256) * SLAB_BYTES;           // behind the buffers of the largest tile
    uint32_t *col_lds = reinterpret_cast<uint32_t *>(smem + AUX_OFF);
    EpiProt<DT> ep;
    ep.st.rdot = T::zero(); ep.st.amax = 0.f;
    ep.col_lds = col_lds; ep.slab0 = tn; ep.slab_step = g.tiles_n; ep.owned = 0;
    ep.col_copies = 4; ep.col_stride = 0;
    {
        const int nslab = K / KE;                      // at least 3 (gemm_fast_eligible)
        int next_own = tn;
        const int owned = (PROT && tn < nslab) ? (nslab - tn + g.tiles_n - 1) / g.tiles_n : 0;
        // column sums: one set of owned * KE words per wave (plain stores, added up by the epilogue)
        ep.col_stride = owned * KE;
        uint32_t *col_mine = col_lds + wave * owned * KE;
        uint32_t *b_lds = col_lds + 4 * owned * KE;
        if (PROT) {
            // the values of b the owned slabs need, straight into LDS (one slab per wave and turn):
            // in place behind the first barrier
            for (int j = wave; j < owned; j += 4) {
                const uint32_t *src = g.b_sum + (long)bz * K + (long)(tn + j * g.tiles_n) * KE + lane;
#pragma unroll
                for (int h = 0; h < KE / 64; ++h)
                    __builtin_amdgcn_global_load_lds((gas_ptr)(src + 64 * h), (las_ptr)(b_lds + j * KE + 64 * h), 4, 0, 0);
            }
        }
        issue_loads(0, 0);
        issue_loads(1, 1);
        // Start as soon as slab 0 is in place: loads complete in order, so "at most the GA + GB
        // loads of slab 1 outstanding" means everything issued before them has landed.  (The
        // barrier inside slab 0 waits for the rest.)
        if constexpr (GA + GB == 16) asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else if constexpr (GA + GB == 12) asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else __syncthreads();
        ldfr(0, 0, 0);
        // own_c: whether the slab can be one that this workgroup reduces (the first slab and the last
        // two: the pass then runs ahead of the slab's MFMAs; the middle slabs have own_slab below)
        auto slab = [&](auto first_c, auto loads_c, auto own_c, int s) __attribute__((always_inline)) {
            constexpr bool LOADS = decltype(loads_c)::value;
            const int buf = s & 1;
            if (PROT && decltype(own_c)::value && s == next_own) {
                if (g.a_given)
                    a_pass<DT, BM, true, true, true, true>(smem + buf * BUF, b_lds + ep.owned * KE, a_rows, col_mine + ep.owned * KE, ep.st,
                                         g.mul24_ok != 0);
                else
                    a_pass<DT, BM, false, true, true, true>(smem + buf * BUF, b_lds + ep.owned * KE, a_rows, col_mine + ep.owned * KE, ep.st,
                                   g.mul24_ok != 0);
                next_own += g.tiles_n;
                ep.owned += 1;
            }
            __builtin_amdgcn_sched_barrier(0);
            ldfr(buf, 1, 1); mfmas(first_c, 0); interleave();
            __builtin_amdgcn_sched_barrier(0);
            ldfr(buf, 2, 0); mfmas(std::false_type{}, 1); interleave();
            __builtin_amdgcn_sched_barrier(0);
            ldfr(buf, 3, 1); mfmas(std::false_type{}, 0); interleave();
            __syncthreads();
            if constexpr (LOADS) {
                step3_loads(s + 2, buf);
            } else {
                ldfr(buf ^ 1, 0, 0);                   // after the last slab: read and never used
                mfmas(std::false_type{}, 1); interleave();
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // A middle slab that this workgroup reduces: the same MFMAs, fragment reads and loads as any
        // other slab, in explicit program order (one group per MFMA, fenced), with one piece of the
        // pass over the slab (gemm_apass.h) behind every MFMA.  The pieces start half a step late, so
        // that the chunks begin() requested have arrived.  Straight-line code of its own: a branch
        // around the pass inside the common slab code keeps it apart from the MFMAs, and the pass
        // then runs while the matrix pipe waits.
        // (With a checksum of A supplied by the caller the column sums and the maximum are formed all
        // the same, under the MFMAs, and not handed on: a second copy of the slab would have to sit
        // behind a branch.)
        auto own_slab = [&](int s) __attribute__((always_inline)) {
            constexpr bool GIVEN = false;
            constexpr int NMF = MI * NI, NLD = GA + GB, LAG = NMF / 2;
            const int buf = s & 1;
            APassSteps<DT, BM, GIVEN> ap;
            __builtin_amdgcn_sched_barrier(0);
            ap.begin(smem + buf * BUF, b_lds + ep.owned * KE, a_rows);
            const uint8_t *ak = a_base + (long)(s + 2) * SLAB_BYTES;
            const uint8_t *bk = b_base + (long)(s + 2) * SLAB_BYTES;
            uint8_t *dA = smem + buf * BUF;
            uint8_t *dB = dA + BM * SLAB_BYTES;
            static_for<0, 4>([&](auto t_c) {
                constexpr int t = decltype(t_c)::value;
                constexpr int set = t & 1, nset = set ^ 1;
                // fragments of the next step: step t + 1 of this slab, or step 0 of the next slab
                const uint8_t *sA = smem + (t < 3 ? buf : buf ^ 1) * BUF;
                const uint8_t *sB = sA + BM * SLAB_BYTES;
                const int sw = ((2 * ((t + 1) & 3) + lh) ^ ((lane >> 1) & 7)) * 16;
                static_for<0, NMF>([&](auto j_c) {
                    constexpr int j = decltype(j_c)::value;
                    constexpr int mi = j / NI, ni = j % NI;
                    acc[mi][ni] = T::mfma(fb[set][ni], fa[set][mi], acc[mi][ni]);
                    if constexpr (j < MI)
                        fa[nset][j] = *reinterpret_cast<const i32x4 *>(sA + (wm * TM + j * 32 + l32) * SLAB_BYTES + sw);
                    else if constexpr (j < MI + NI)
                        fb[nset][j - MI] = *reinterpret_cast<const i32x4 *>(sB + (wn * TN + (j - MI) * 32 + l32) * SLAB_BYTES + sw);
                    if constexpr (t == 3) {
                        constexpr int l0 = j * NLD / NMF, l1 = (j + 1) * NLD / NMF;
                        static_for<l0, l1>([&](auto l_c) {
                            constexpr int l = decltype(l_c)::value;
                            if constexpr (l < GA)
                                __builtin_amdgcn_global_load_lds((gas_ptr)(ak + a_off[l]), (las_ptr)(dA + (4 * l + wave) * 8 * SLAB_BYTES), 16, 0, 0);
                            else
                                __builtin_amdgcn_global_load_lds((gas_ptr)(bk + b_off[l - GA]), (las_ptr)(dB + (4 * (l - GA) + wave) * 8 * SLAB_BYTES), 16, 0, 0);
                        });
                    }
                    ap.template piece<t * NMF + j - LAG>();
                    __builtin_amdgcn_sched_barrier(0);
                });
                if constexpr (t == 2) __syncthreads();
            });
            static_for<4 * NMF - LAG, 4 * NMF>([&](auto k_c) { ap.template piece<decltype(k_c)::value>(); });
            ap.end(col_mine + ep.owned * KE, ep.st);
            __builtin_amdgcn_sched_barrier(0);
            next_own += g.tiles_n;
            ep.owned += 1;
        };
        typedef std::false_type never_own;
        typedef std::true_type maybe_own;
        slab(std::true_type{}, std::true_type{}, maybe_own{}, 0);
        // the middle slabs: runs of slabs that are not this workgroup's, each followed by one that is
        int s = 1;
        const int mid_end = nslab - 2;
        // (loops and straight-line code only: an if / else with MFMAs in both arms would move the
        // accumulators out of the accumulation registers)
        if constexpr (PROT) {
            while (next_own < mid_end) {                   // next_own >= s here
                for (; s < next_own; ++s) slab(std::false_type{}, std::true_type{}, never_own{}, s);
                own_slab(s);
                ++s;
            }
        }
        for (; s < mid_end; ++s) slab(std::false_type{}, std::true_type{}, never_own{}, s);
        for (; s < nslab; ++s) slab(std::false_type{}, std::false_type{}, maybe_own{}, s);
    }
    __syncthreads();
    gemm_epilogue<DT, BM, BN, PROT>(g, acc, smem, m0, n0, bz, ep);
}

// Workgroup -> tile inside a region of tiles_m x tiles_n tiles: consecutive ids of one XCD
// (workgroups are dealt to the 8 XCDs round-robin) walk GROUP_M tile rows, then the next column,
// so the workgroups that share an L2 work on a compact group of tiles.
__device__ __forceinline__ void map_tile(int bid, int nb, int tiles_m, int tiles_n, int *tm, int *tn)
{
    constexpr int GROUP_M = 4;          // measured against 2, 3, 6, 8, 16: best or equal on every Linear shape
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
// big_rows rows, 128 x 256 tiles the rest; how many of each is chosen by playing the dispatch
// through (choose_big_rows).  (600 big tiles on 256 CUs would be three rounds for 2.34 rounds
// of work.)
template <int DT, bool PROT>
__global__ __launch_bounds__(256) void gemm_fast_kernel(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // Persistent workgroups: one per compute unit, each walks the tile list with the grid's stride.
    // The 128-row tiles come first in the list: the compute units that start with one are half a
    // tile ahead of the others from then on, so the two groups store their tiles of C at different
    // times (a round of the machine that stores in step asks for tens of MB at once) and draw on
    // the matrix pipes at different times.  Measured on 12608 x 3072 x 768: 63 -> 60.5 us.
    const int per_item = g.n_small + g.n_big;
    const int total = per_item * g.batch;
    for (int t = blockIdx.x; t < total; t += gridDim.x) {
        const int bz = t / per_item, bid = t - bz * per_item;
        int tm, tn;
        if (bid >= g.n_small) {
            map_tile(bid - g.n_small, g.n_big, g.tiles_m_big, g.tiles_n, &tm, &tn);
            fast_tile<DT, 256, 256, PROT>(g, smem, tm * 256, tn * 256, bz, tn);
        } else {
            map_tile(bid, g.n_small, g.tiles_m_small, g.tiles_n, &tm, &tn);
            fast_tile<DT, 128, 256, PROT>(g, smem, g.tiles_m_big * 256 + tm * 128, tn * 256, bz, tn);
        }
        // the epilogue's last reads of LDS precede the next tile's first writes
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
}

// ------------------------------------------------------------------------------------------
// How many tile rows get 256-row tiles (the rest of M gets 128-row tiles).  Workgroups are
// dispatched in index order to whichever CU is free, one per CU; a 128 x 256 tile takes about
// 0.62 of the time of a 256 x 256 tile (measured), not half: its main loop waits on the same
// load latency per slab.  A few candidate splits are played through with those two costs and
// the one that finishes first wins; the result is remembered per shape.
static double play_schedule(int big_rows, int M, int tiles_n, int batch, int ncu)
{
    const int rest = M - big_rows * 256;
    const long nb = (long)big_rows * tiles_n, ns = (long)(rest > 0 ? (rest + 127) / 128 : 0) * tiles_n;
    std::priority_queue<double, std::vector<double>, std::greater<double>> cu;
    for (int i = 0; i < ncu; ++i) cu.push(0.0);
    double end = 0.0;
    for (int z = 0; z < batch; ++z)
        for (long t = 0; t < nb + ns; ++t) {
            const double f = cu.top() + (t < ns ? 0.62 : 1.0);     // dispatch order: the half-height tiles first
            cu.pop();
            cu.push(f);
            if (f > end) end = f;
        }
    return end;
}

static int choose_big_rows(int M, int tiles_n, int batch, int ncu)
{
    struct Memo { int M, tiles_n, batch, ncu, big_rows; };
    static Memo memo[16];
    static int memo_n = 0;
    static std::mutex memo_lock;                 // contexts may be driven from different host threads
    std::lock_guard<std::mutex> hold(memo_lock);
    for (int i = 0; i < memo_n; ++i)
        if (memo[i].M == M && memo[i].tiles_n == tiles_n && memo[i].batch == batch && memo[i].ncu == ncu)
            return memo[i].big_rows;
    const int rows_all_big = (M + 255) / 256;
    const long per_row = (long)tiles_n * batch;
    const long total_big = rows_all_big * per_row;
    int cand[4], nc = 0;
    cand[nc++] = rows_all_big;                                   // big tiles only
    cand[nc++] = 0;                                              // half-height tiles only
    long whole = (total_big / ncu) * ncu / per_row;              // whole rounds of big tiles
    if (whole > rows_all_big) whole = rows_all_big;
    cand[nc++] = (int)whole;
    const long fewer = whole - (ncu + per_row - 1) / per_row;    // one round fewer
    if (fewer > 0) cand[nc++] = (int)fewer;
    int best = cand[0];
    double best_t = play_schedule(cand[0], M, tiles_n, batch, ncu);
    for (int i = 1; i < nc; ++i) {
        const double t = play_schedule(cand[i], M, tiles_n, batch, ncu);
        if (t < best_t - 1e-9) { best_t = t; best = cand[i]; }
    }
    Memo m = {M, tiles_n, batch, ncu, best};
    memo[memo_n < 16 ? memo_n++ : (M + tiles_n) & 15] = m;
    return best;
}

template <int DT, bool PROT>
static hipError_t launch_fast_one(GemmArgs &g, int batch, hipStream_t st)
{
    constexpr int smem_main = 2 * (256 + 256) * SLAB_BYTES;
    constexpr int smem_max = 160 * 1024;
    auto kern = gemm_fast_kernel<DT, PROT>;
    hipError_t e = ensure_max_lds(reinterpret_cast<const void *>(kern), smem_max);
    if (e != hipSuccess) return e;
    const int num_cu = device_cu_count(&e);
    if (e != hipSuccess) return e;
    g.tiles_n = (g.N + 255) / 256;
    const int big_rows = choose_big_rows(g.M, g.tiles_n, batch, num_cu);
    g.tiles_m_big = big_rows;
    g.n_big = big_rows * g.tiles_n;
    const int rest = g.M - big_rows * 256;
    g.tiles_m_small = rest > 0 ? (rest + 127) / 128 : 0;
    g.tiles_m = g.tiles_m_big + g.tiles_m_small;
    g.n_small = g.tiles_m_small * g.tiles_n;
    g.batch = batch;
    const long total = (long)(g.n_big + g.n_small) * batch;
    if (total > 0x7FFFFFFFL) return hipErrorInvalidValue;
    dim3 grid((unsigned)(total < num_cu ? total : num_cu), 1, 1);
    size_t smem = smem_main;
    if (PROT) {
        const int ke = SLAB_BYTES / Traits<DT>::ES;
        smem += apass_lds_bytes_per_wave(DT, g.K / ke, g.tiles_n);
        if (smem > (size_t)smem_max) return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, g);
    return hipGetLastError();
}

bool gemm_fast_eligible(int dt, int M, int N, int K, bool transB, long lda, long ldb)
{
    const int ke = SLAB_BYTES / elem_size(dt);
    // whole slabs, at least three of them (the main loop is peeled), and 32-bit row offsets
    // inside a tile
    // (int8: N < 65536 keeps |b| <= 128 N below 2^23, which the pass over A's slabs relies on here)
    return transB && (K % ke) == 0 && K >= 3 * ke && M >= 512 && N >= 512 && (dt != DT_I8 || N < 65536) &&
           lda * elem_size(dt) < (1L << 23) && ldb * elem_size(dt) < (1L << 23) &&
           // what the pass over A's slabs keeps per tile fits behind the operand buffers (protected or
           // not: the tile shape of a problem does not depend on the mode)
           2 * (256 + 256) * SLAB_BYTES + apass_lds_bytes_per_wave(dt, K / ke, (N + 255) / 256) <= 160 * 1024;
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
