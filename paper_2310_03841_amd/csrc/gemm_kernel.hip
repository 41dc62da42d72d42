// Protected GEMM kernel for gfx950, general shapes: C = A * B with the observed row / column
// sums of C taken from the accumulators in the epilogue and the input-side checksums of A
// taken from the operand slabs while they are resident in LDS.
//
// Method: classic row/column ABFT as cited by the paper (Sec. I, Sec. II-B), with the paper's
// epilogue fusion of the output checksum (Sec. IV-C memory paragraph; Sec. V "Optimizations"
// (2)).
//
// Tiling: one workgroup of 4 waves computes a BM x BN tile; each wave owns a
// (BM/2) x (BN/2) sub-tile as 32x32 MFMA blocks.  K advances in slabs of 128
// bytes per row, double-buffered in LDS.  LDS rows are 128 bytes, stored as
// eight 16-byte chunks with chunk index XOR (row & 7) so that both the
// row-contiguous writes and the MFMA operand reads are bank-conflict free.
// Rows of A past M and the tail of a ragged K are zero-filled in LDS.
#include "abft_device.h"
#include "gemm_args.h"
#include "gemm_epilogue.h"

namespace abft {


template <int DT, int BM, int BN, bool PROT, bool TRANSB>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g)
{
    using T = Traits<DT>;
    typedef typename T::accv_t accv_t;
    constexpr int ES = T::ES;
    constexpr int CE = 16 / ES;                  // elements per 16-byte chunk
    constexpr int KE = SLAB_BYTES / ES;          // elements of K per slab
    constexpr int TM = BM / 2, TN = BN / 2;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int PA = BM / 32, PB = BN / 32;    // chunks per thread per slab
    constexpr int BUF = (BM + BN) * SLAB_BYTES;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform by construction
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    const int bz = blockIdx.z;

    const int tm_idx = blockIdx.x % g.tiles_m;
    const int tn_idx = blockIdx.x / g.tiles_m;
    const int m0 = tm_idx * BM, n0 = tn_idx * BN;
    const int M = g.M, N = g.N, K = g.K;

    const uint8_t *Ab = g.A + (long)bz * g.sA * ES;
    const uint8_t *Bb = g.B + (long)bz * g.sB * ES;

    // ---- per-thread row sources: chunk column c of rows r0 + 32 p
    const int c = tid & 7, r0 = tid >> 3;
    const uint8_t *asrc[PA];
    const uint8_t *bsrc[PB];
    bool btail[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        int r = m0 + r0 + 32 * p;
        asrc[p] = r < M ? Ab + (long)r * g.lda * ES : nullptr;     // rows past M are zero-filled
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int r = n0 + r0 + 32 * p;
        btail[p] = r >= N;                           // rows of the B tile past N are zero-filled
        bsrc[p] = (TRANSB && r < N) ? Bb + (long)r * g.ldb * ES : nullptr;
    }
    const bool tile_has_btail = (n0 + BN > N);

    // ---- accumulators
    accv_t acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mi][ni][i] = T::zero();
    bool mact[MI], nact[NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) mact[mi] = (m0 + wm * TM + mi * 32) < M;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) nact[ni] = (n0 + wn * TN + ni * 32) < N;

    // Two register sets: the slab after next is already on its way from memory while the next
    // one is written to LDS (small problems are a chain of memory latencies otherwise).
    struct SlabRegs { i32x4 a[PA], b[PB], bnn[PB]; };
    SlabRegs R0, R1;
    const int nslab = (K + KE - 1) / KE;
    const bool ragged_k = (K % KE) != 0;

    auto load_rowmajor = [&](const uint8_t *const *src, i32x4 *regs, int P, int k0, bool tail) {
        const int kb = k0 + c * CE;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            i32x4 v = {0, 0, 0, 0};
            if (src[p] != nullptr && (!tail || kb < K)) {
                v = *reinterpret_cast<const i32x4 *>(src[p] + (long)kb * ES);
                if (tail && kb + CE > K) v = mask_chunk(v, (K - kb) * ES);
            }
            regs[p] = v;
        }
    };
    auto store_rowmajor = [&](uint8_t *dst, const i32x4 *regs, int P, const bool *only) {
        const int sw = (c ^ (r0 & 7)) * 16;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (only == nullptr || only[p])
                *reinterpret_cast<i32x4 *>(dst + (r0 + 32 * p) * SLAB_BYTES + sw) = regs[p];
        }
    };
    // B stored K x N: chunks run along n; they are transposed while written to LDS.
    constexpr int NCH = BN / CE;
    auto load_b_nn = [&](int k0, i32x4 *bnn) {
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            int q = tid + 256 * p;
            int nch = q % NCH, kk = q / NCH;
            int k = k0 + kk, nst = n0 + nch * CE;
            i32x4 v = {0, 0, 0, 0};
            if (k < K && nst < N) v = *reinterpret_cast<const i32x4 *>(Bb + ((long)k * g.ldb + nst) * ES);
            bnn[p] = v;
        }
    };
    auto store_b_nn = [&](uint8_t *dst, const i32x4 *bnn) {
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            int q = tid + 256 * p;
            int nch = q % NCH, kk = q / NCH;
            int kc = kk / CE, ke = kk % CE;
#pragma unroll
            for (int e = 0; e < CE; ++e) {
                int nl = nch * CE + e;
                if (n0 + nl < N) {
                    uint8_t *d = dst + nl * SLAB_BYTES + ((kc ^ (nl & 7)) * 16) + ke * ES;
                    if (ES == 2) {
                        uint32_t w = (uint32_t)bnn[p][e >> 1];
                        *reinterpret_cast<uint16_t *>(d) = (uint16_t)((e & 1) ? (w >> 16) : (w & 0xFFFFu));
                    } else {
                        uint32_t w = (uint32_t)bnn[p][e >> 2];
                        *d = (uint8_t)(w >> (8 * (e & 3)));
                    }
                }
            }
        }
    };

    auto load_slab = [&](int s, SlabRegs &R) __attribute__((always_inline)) {
        if (s >= nslab) return;
        const int k0 = s * KE;
        const bool tail = ragged_k && (s == nslab - 1);
        load_rowmajor(asrc, R.a, PA, k0, tail);
        if (TRANSB) {
            load_rowmajor(bsrc, R.b, PB, k0, tail);
        } else {
            load_b_nn(k0, R.bnn);
            if (tile_has_btail) load_rowmajor(bsrc, R.b, PB, k0, tail);
        }
    };
    auto store_slab = [&](int s, const SlabRegs &R) __attribute__((always_inline)) {
        if (s >= nslab) return;
        uint8_t *sA = smem + (s & 1) * BUF;
        uint8_t *sB = sA + BM * SLAB_BYTES;
        store_rowmajor(sA, R.a, PA, nullptr);
        if (TRANSB) {
            store_rowmajor(sB, R.b, PB, nullptr);
        } else {
            store_b_nn(sB, R.bnn);
            if (tile_has_btail) store_rowmajor(sB, R.b, PB, btail);
        }
    };
    auto compute = [&](int buf) {
        const uint8_t *sA = smem + buf * BUF;
        const uint8_t *sB = sA + BM * SLAB_BYTES;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
            const int sw = ((2 * s4 + lh) ^ (lane & 7)) * 16;
            i32x4 af[MI], bf[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[mi] = *reinterpret_cast<const i32x4 *>(sA + (wm * TM + mi * 32 + l32) * SLAB_BYTES + sw);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bf[ni] = *reinterpret_cast<const i32x4 *>(sB + (wn * TN + ni * 32 + l32) * SLAB_BYTES + sw);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    if (mact[mi] && nact[ni]) acc[mi][ni] = T::mfma(bf[ni], af[mi], acc[mi][ni]);
        }
    };

    // Protected tiles reduce the slabs of A they own (slab s belongs to tile column s mod
    // tiles_n) while those are resident: see gemm_apass.h.
    uint32_t *col_lds = reinterpret_cast<uint32_t *>(smem + 2 * BUF);
    EpiProt<DT> ep;
    ep.st.rdot = T::zero(); ep.st.amax = 0.f;
    ep.col_lds = col_lds; ep.slab0 = tn_idx; ep.slab_step = g.tiles_n; ep.owned = 0;
    ep.col_copies = 1; ep.col_stride = 0;
    int next_own = tn_idx;
    const int owned = (PROT && tn_idx < nslab) ? (nslab - tn_idx + g.tiles_n - 1) / g.tiles_n : 0;
    uint32_t *b_lds = col_lds + owned * KE;
    if (PROT) {
        // zeros for the column sums and the values of b the owned slabs need (zero beyond K);
        // both are in place behind the first barrier
        for (int t = tid; t < owned * KE; t += 256) {
            const int kk = (tn_idx + (t / KE) * g.tiles_n) * KE + (t % KE);
            col_lds[t] = 0u;
            b_lds[t] = kk < K ? g.b_sum[(long)bz * K + kk] : 0u;
        }
    }

    // ---- main loop: global -> registers -> LDS, two LDS buffers, one barrier per slab.  While
    // slab s is multiplied, slab s + 1 goes from its register set to the other LDS buffer and the
    // loads of slab s + 3 are issued into the set that has just been emptied (slab s + 2 is in
    // flight in the other set).
    auto one_slab = [&](int s, SlabRegs &Rnext, SlabRegs & /*Rafter*/) __attribute__((always_inline)) {
        if (PROT && s == next_own) {
            if (g.a_given)
                a_pass<DT, BM, true>(smem + (s & 1) * BUF, b_lds + ep.owned * KE, BM, col_lds + ep.owned * KE, ep.st,
                                     g.mul24_ok != 0);
            else
                a_pass<DT, BM>(smem + (s & 1) * BUF, b_lds + ep.owned * KE, BM, col_lds + ep.owned * KE, ep.st,
                               g.mul24_ok != 0);
            next_own += g.tiles_n;
            ep.owned += 1;
        }
        compute(s & 1);
        store_slab(s + 1, Rnext);
        load_slab(s + 3, Rnext);
        __syncthreads();
    };
    load_slab(0, R0);
    load_slab(1, R1);
    store_slab(0, R0);
    load_slab(2, R0);
    __syncthreads();
    for (int s = 0; s < nslab; s += 2) {
        one_slab(s, R1, R0);
        if (s + 1 < nslab) one_slab(s + 1, R0, R1);
    }

    // ---- epilogue
    gemm_epilogue<DT, BM, BN, PROT>(g, acc, smem, m0, n0, bz, ep);
}

// ------------------------------------------------------------------------------------------
template <int DT, int BM, int BN, bool PROT, bool TRANSB>
static hipError_t launch_one(const GemmArgs &g, int batch, hipStream_t st)
{
    constexpr int smem_main = 2 * (BM + BN) * SLAB_BYTES;
    constexpr int smem_max = smem_main + (PROT ? (4096 + SLAB_BYTES) * 8 : 0);
    auto kern = gemm_kernel<DT, BM, BN, PROT, TRANSB>;
    if (smem_max > 48 * 1024) {
        hipError_t e = ensure_max_lds(reinterpret_cast<const void *>(kern), smem_max);
        if (e != hipSuccess) return e;
    }
    size_t smem = smem_main;
    if (PROT) {
        const int ke = SLAB_BYTES / Traits<DT>::ES;
        smem += apass_lds_bytes(DT, (g.K + ke - 1) / ke, g.tiles_n);
        if (smem > (size_t)smem_max) return hipErrorInvalidValue;
    }
    dim3 grid((unsigned)(g.tiles_m * g.tiles_n), 1, (unsigned)batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, g);
    return hipGetLastError();
}

template <int DT, int BM, int BN>
static hipError_t launch_cfg(bool protect, bool transB, GemmArgs &g, int batch, hipStream_t st)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    if (protect) return transB ? launch_one<DT, BM, BN, true, true>(g, batch, st)
                               : launch_one<DT, BM, BN, true, false>(g, batch, st);
    return transB ? launch_one<DT, BM, BN, false, true>(g, batch, st)
                  : launch_one<DT, BM, BN, false, false>(g, batch, st);
}

void gemm_tile_shape(int dt, const Shape &s, int *tm, int *tn)
{
    if (gemm_item_eligible(dt, s, false)) {          // one workgroup per batch item
        *tm = s.M;
        *tn = s.N;
        return;
    }
    if (gemm_fast_eligible(dt, s.M, s.N, s.K, s.transB != 0, s.lda, s.ldb)) {
        gemm_fast_tile(tm, tn);
        return;
    }
    *tm = 128;
    *tn = 128;
}

hipError_t launch_gemm(int dt, bool protect, bool stored_sums, const void *A, const void *B, void *C,
                       const Shape &s, const Workspace &w, const InjectArm &arm, hipStream_t st)
{
    if (!protect && !w.bias && gemm_item_eligible(dt, s, false))
        return launch_gemm_item(dt, false, false, false, A, B, C, s, w, nullptr, arm, st);
    GemmArgs g;
    g.A = (const uint8_t *)A;
    g.B = (const uint8_t *)B;
    g.C = (uint8_t *)C;
    g.M = s.M; g.N = s.N; g.K = s.K;
    g.lda = s.lda; g.ldb = s.ldb; g.ldc = s.ldc;
    g.sA = s.sA; g.sB = s.sB; g.sC = s.sC;
    g.inj_b = arm.batch; g.inj_row = arm.row; g.inj_col = arm.col; g.inj_bit = arm.bit;
    g.cc_obs = w.cc_obs; g.rc_obs = w.rc_obs; g.rc_pred = w.rc_pred;
    g.a_sum = w.a_sum; g.a_max = w.a_max; g.b_sum = w.b_sum;
    g.bias = w.bias;
    g.cc_sto = (protect && stored_sums && dt != DT_I8) ? w.cc_sto : nullptr;
    g.rc_sto = g.cc_sto ? w.rc_sto : nullptr;
    g.c_max = g.cc_sto ? w.c_max : nullptr;
    g.a_given = (protect && w.a_given) ? 1 : 0;
    g.mul24_ok = s.N < 65536 ? 1 : 0;            // |b| <= 128 N
    g.tiles_m = g.tiles_n = g.n_big = g.tiles_m_big = g.tiles_m_small = 0;
    g.n_small = 0; g.batch = s.batch;
    const bool tb = s.transB != 0;
    if (gemm_fast_eligible(dt, s.M, s.N, s.K, tb, s.lda, s.ldb)) return launch_gemm_fast(dt, protect, g, s.batch, st);
    switch (dt) {
    case DT_I8:   return launch_cfg<DT_I8, 128, 128>(protect, tb, g, s.batch, st);
    case DT_BF16: return launch_cfg<DT_BF16, 128, 128>(protect, tb, g, s.batch, st);
    case DT_F16:  return launch_cfg<DT_F16, 128, 128>(protect, tb, g, s.batch, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace abft
