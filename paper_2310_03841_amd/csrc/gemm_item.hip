// Protected GEMM for batches of small problems (the per-head attention products Q K^T and
// attn V): one workgroup owns a whole batch item, so every checksum of the scheme
// (Sec. III-B.1 "Checksums") is formed and checked inside that workgroup -- no atomics on
// global memory, no separate pass over B, no finish kernel.
//
// Per item: B is brought into LDS once and stays (as rows n of K-contiguous 128-byte slabs, the
// layout the MFMA fragment reads want; a B stored K x N is transposed on the way in).  b = B e
// and max|B| are taken from that copy (for a B stored K x N: from the registers of the
// transposing load).  A streams through a ring of LDS buffers in blocks of 32 or 64 rows, filled
// by direct-to-LDS loads that a fifth wave issues several blocks ahead.  That wave does nothing
// else: the memory counter of a wave counts its loads and its stores in one sequence, so a wave
// that stores C cannot wait for a load without also waiting for its stores to be acknowledged;
// with the roles split the four computing waves never wait on memory at all.  (Where all of A
// fits in LDS it is fetched at the start of the item and the fifth wave is left out.)  From each
// resident block come its share of a = e^T A, the row prediction A b and max|A|, from the
// accumulators the observed row and column sums (before rounding; Sec. IV-C memory paragraph,
// Sec. V "Optimizations" (2)), and C leaves through a wave-private LDS stage as row-contiguous
// segments.  When the last block is done the column prediction a B is formed from the resident
// B, both pairs are compared (equality for int8, tolerance for floating point; Sec. III-B.1
// item (2)), and the vectors, flags and counts are written.
//
// These products are bound by memory traffic (about 39 flop per byte at 197 x 197 x 64), so the
// design goal is streaming: few dependent round trips per item, row segments that the L2 can
// merge into whole lines, and nothing read twice from memory.
#include "abft_device.h"
#include "gemm_args.h"
#include "gemm_apass.h"
#include "gemm_epilogue.h"

namespace abft {

constexpr int ITEM_MAX_SLABS = 5;          // K * element size <= 640 bytes
constexpr int ITEM_MAX_M = 1024;
constexpr int ITEM_MIN_BATCH = 64;         // fewer items leave most compute units without work
constexpr int ITEM_MAX_BLOCKS = 1024;      // workgroups; items beyond are taken in turn
constexpr int ITEM_GROUP = 16;             // workgroups per first-level ticket
constexpr int ITEM_STAGE_ROW = 36;         // words per staged row of a 32 x 32 block (32 + pad)
constexpr int ITEM_STAGE_WAVE = 32 * ITEM_STAGE_ROW * 4;
// two 16-bit integers in one register, and the same 32 bits as a word (for moves between lanes)
typedef short item_s16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ item_s16x2 item_pair(int w) { return item_s16x2{(short)(w & 0xFFFF), (short)(w >> 16)}; }
__device__ __forceinline__ int item_word(item_s16x2 v)
{
    return (int)(((uint32_t)(uint16_t)v[1] << 16) | (uint32_t)(uint16_t)v[0]);
}
constexpr int ITEM_LDS_LIMIT = 160 * 1024;
constexpr int ITEM_THREADS = 320;          // four computing waves and the loading wave
constexpr int ITEM_MAX_STAGES = 8;

typedef const __attribute__((address_space(1))) void *item_gas_ptr;
typedef __attribute__((address_space(3))) void *item_las_ptr;

// Workgroup barrier over LDS traffic only.  The waves meet to exchange data through LDS; a full
// barrier would also wait until every store of C issued so far has been acknowledged (and, in
// the loading wave, until every block in flight has landed), which is the latency this kernel
// is built to hide.  Data that arrives in LDS by direct loads is waited for explicitly.
__device__ __forceinline__ void item_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// s_waitcnt vmcnt(n) for a run-time n (the instruction takes an immediate).
__device__ __forceinline__ void item_wait_vmcnt(int n)
{
#define ITEM_W(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
    switch (n) {
        ITEM_W(0) ITEM_W(1) ITEM_W(2) ITEM_W(3) ITEM_W(4) ITEM_W(5) ITEM_W(6) ITEM_W(7)
        ITEM_W(8) ITEM_W(9) ITEM_W(10) ITEM_W(11) ITEM_W(12) ITEM_W(13) ITEM_W(14) ITEM_W(15)
        ITEM_W(16) ITEM_W(17) ITEM_W(18) ITEM_W(19) ITEM_W(20) ITEM_W(21) ITEM_W(22) ITEM_W(23)
        ITEM_W(24) ITEM_W(25) ITEM_W(26) ITEM_W(27) ITEM_W(28) ITEM_W(29) ITEM_W(30) ITEM_W(31)
        ITEM_W(32) ITEM_W(33) ITEM_W(34) ITEM_W(35) ITEM_W(36) ITEM_W(37) ITEM_W(38) ITEM_W(39)
        ITEM_W(40) ITEM_W(41) ITEM_W(42) ITEM_W(43) ITEM_W(44) ITEM_W(45) ITEM_W(46) ITEM_W(47)
        ITEM_W(48) ITEM_W(49) ITEM_W(50) ITEM_W(51) ITEM_W(52) ITEM_W(53) ITEM_W(54) ITEM_W(55)
        ITEM_W(56) ITEM_W(57) ITEM_W(58) ITEM_W(59) ITEM_W(60) ITEM_W(61) ITEM_W(62) ITEM_W(63)
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
#undef ITEM_W
}

struct ItemArgs {
    const uint8_t *A, *B;
    uint8_t *C;
    int M, N, K, batch;
    long lda, ldb, ldc, sA, sB, sC;               // elements
    int nslab;                                    // 128-byte slabs that cover a row of K
    int nch;                                      // 16-byte chunks of a row that hold data
    int ksteps;                                   // MFMA steps over K (32 bytes of K per row each)
    int NB;                                       // blocks of 32 columns
    int nrb;                                      // blocks of rows
    int stages;                                   // LDS buffers for blocks of A: a ring of 2..8, or one per block (nrb)
    int inj_b, inj_row, inj_col, inj_bit;         // armed accumulator flip (inj_b < 0: none)
    int mul24_ok;
    int b16_ok;                                   // int8: |b| < 2^15 (N <= 255): the row dots take 16-bit pairs
    int cached_b;                                 // take b and max|B| from b_sum / b_max instead of forming them
    // protected launches: everything below is written with plain stores, item by item
    uint32_t *cc_obs, *rc_obs, *rc_pred, *a_sum, *a_max, *b_sum, *b_max, *cc_pred, *s_pred;
    uint32_t *cc_sto, *rc_sto;                    // sums of C as stored (after rounding), on request (floating point)
    float *maxabs, *tau;
    float tau_override, tau_override_cols;
    uint8_t *row_flag, *col_flag;
    uint32_t *counts;
    uint32_t *ticket;                             // [3]: ticket, flagged rows, flagged cols (self-cleaning)
    uint32_t *group_ticket;                       // [ITEM_MAX_BLOCKS / ITEM_GROUP] (self-cleaning)
};

// Slabs of K a configuration takes: the column sums of A stay in registers over all row blocks
// of an item (16 bytes of columns per slab and thread), so wide tiles leave room for few.
__host__ __device__ constexpr int item_max_slabs(int wm, int tpw) { return wm == 2 ? ITEM_MAX_SLABS : (tpw <= 2 ? 3 : 2); }

// LDS of a workgroup: B, `stages` buffers for blocks of A, the waves' output stages, vectors.
__host__ __device__ inline size_t item_lds_bytes(int dt, int wm, int stages, int M, int N, int K, bool sto)
{
    const int es = elem_size(dt), ke = SLAB_BYTES / es;
    const int nslab = (K * es + SLAB_BYTES - 1) / SLAB_BYTES;
    const int bmr = 32 * wm;
    const int Nr = (N + 31) / 32 * 32, Mr = (M + bmr - 1) / bmr * bmr;
    size_t b = (size_t)nslab * Nr * SLAB_BYTES + (size_t)stages * nslab * bmr * SLAB_BYTES + 4 * ITEM_STAGE_WAVE;
    b += ((size_t)2 * nslab * ke + 2 * Mr + Nr + 24) * 4;
    if (sto) b += ((size_t)Mr + Nr) * 4;          // stored-side sums
    return b;
}

// Depth of the ring.  A depth of all the item's row blocks means A is resident as a whole and
// the computing waves run through the blocks without meeting.  Otherwise: as deep as half the
// LDS of a compute unit allows (two workgroups per unit), else as deep as the whole allows; the
// loading wave waits with an immediate count, so (stages - 2) blocks' worth of load
// instructions must stay below 64.  0: does not fit.
__host__ inline int item_stages(int dt, int wm, int M, int N, int K, bool sto)
{
    const int es = elem_size(dt);
    const int nslab = (K * es + SLAB_BYTES - 1) / SLAB_BYTES;
    const int ql = 4 * wm * nslab;
    int smax = 2 + 63 / ql;
    if (smax > ITEM_MAX_STAGES) smax = ITEM_MAX_STAGES;
    const size_t fixed = item_lds_bytes(dt, wm, 0, M, N, K, sto);
    const size_t abuf = (size_t)nslab * 32 * wm * SLAB_BYTES;
    const int nrb = (M + 32 * wm - 1) / (32 * wm);
    const size_t budgets[2] = {(size_t)ITEM_LDS_LIMIT / 2, (size_t)ITEM_LDS_LIMIT};
    for (int i = 0; i < 2; ++i) {
        if (fixed >= budgets[i]) continue;
        long st = (long)((budgets[i] - fixed) / abuf);
        if (st >= nrb) return nrb;               // all of A resident: no ring, no barriers per block
        if (st > smax) st = smax;
        if (st >= (i == 0 ? 3 : 2)) return (int)st;
    }
    return 0;
}

// WM x WN waves; a row block is 32 WM rows; wave (wm, wn) owns the 32-column blocks
// wn, wn + WN, ... (TPW of them at most) of its 32 rows.
// RES: every row block of an item has its own LDS buffer (stages == nrb).  Then all of A is
// fetched at the start of the item, by the four computing waves themselves, and the loading
// wave is left out: with four waves per workgroup two workgroups share a compute unit without
// their waves competing for the registers of one SIMD.
// STO (floating point, protected): also the row / column sums of the values as they are stored.
template <int DT, int WM, int TPW, bool PROT, bool TRANSB, bool RES, bool STO>
__global__ __launch_bounds__(RES ? 256 : ITEM_THREADS) void gemm_item_kernel(ItemArgs g)
{
    constexpr int NT = RES ? 256 : ITEM_THREADS;
    using T = Traits<DT>;
    typedef typename T::acc_t acc_t;
    typedef typename T::accv_t accv_t;
    constexpr int ES = T::ES, OS = T::OS;
    constexpr int CE = 16 / ES;                  // elements per 16-byte chunk
    constexpr int KE = SLAB_BYTES / ES;          // elements of K per slab
    constexpr int WN = 4 / WM, BMr = 32 * WM;
    constexpr int MAXS = item_max_slabs(WM, TPW);   // slabs of K this configuration takes

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = !RES && wave == 4;       // waves 0..3 compute, wave 4 streams A
    const int wm = (wave & 3) / WN, wn = (wave & 3) % WN;
    const int l32 = lane & 31, lh = lane >> 5;
    const int c8 = tid & 7, rg = tid >> 3;       // loader / reducer view: chunk c8 of row rg (+ 32 p)
    const int M = g.M, N = g.N, K = g.K;
    const int nslab = g.nslab, NB = g.NB;
    const int Nr = NB * 32, Mr = g.nrb * BMr;
    const int kbytes = K * ES;

    uint8_t *sB = smem;
    uint8_t *sA0 = sB + (size_t)nslab * Nr * SLAB_BYTES;
    const int abuf = nslab * BMr * SLAB_BYTES;
    const int S = g.stages;
    uint8_t *stage = sA0 + S * abuf + (wave & 3) * ITEM_STAGE_WAVE;
    uint32_t *a_lds = reinterpret_cast<uint32_t *>(sA0 + S * abuf + 4 * ITEM_STAGE_WAVE);
    uint32_t *b_lds = a_lds + nslab * KE;
    uint32_t *rcobs = b_lds + nslab * KE;
    uint32_t *rcpred = rcobs + Mr;
    uint32_t *ccobs = rcpred + Mr;
    uint32_t *rcsto = ccobs + Nr + 24;           // STO: [Mr], then ccsto [Nr]
    uint32_t *ccsto = rcsto + Mr;
    uint32_t *misc = ccobs + Nr;                 // [24]: 0..3 max|A| per wave, 4..7 max|B|, 8..11 a.b partials,
                                                 // 16..23 flagged rows / columns per wave

    auto wave_sync = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    unsigned nr_w = 0, nc_w = 0;                 // flagged rows / columns seen by this wave

    // The ring starts as zeros: chunk positions beyond K are never loaded and must read as zero.
    for (int q = tid; q < S * abuf / 16; q += NT)
        reinterpret_cast<i32x4 *>(sA0)[q] = i32x4{0, 0, 0, 0};
    item_barrier();
    const int QL = 4 * WM * nslab;               // load instructions per block of A
    const bool resident = RES || S >= g.nrb;     // every block of the item has its own buffer
    const int lrow = lane >> 3, lchunk = (lane & 7) ^ lrow;
    const int tail_chunk = (kbytes & 15) ? g.nch - 1 : -1;      // chunk that ends inside its 16 bytes

    for (int bz = blockIdx.x; bz < g.batch; bz += gridDim.x) {
        const uint8_t *Ab = g.A + (long)bz * g.sA * ES;
        const uint8_t *Bb = g.B + (long)bz * g.sB * ES;
        uint8_t *Cb = g.C + (long)bz * g.sC * OS;

        // Block blk of A into its ring buffer: one wave instruction fills 8 rows of 128 bytes;
        // lane l lands in row l >> 3, slot l & 7 and fetches chunk (l & 7) ^ (l >> 3), so that
        // slot = chunk ^ (row & 7).  Rows past M (also whole blocks past the last one, which
        // keep the number of loads in flight constant) fetch the last row: nothing of them is
        // used.
        auto issue_block = [&](int blk) __attribute__((always_inline)) {
            uint8_t *slot = sA0 + (blk % S) * abuf;
            for (int s2 = 0; s2 < nslab; ++s2) {
                const int ch = s2 * 8 + lchunk;
#pragma unroll
                for (int g8 = 0; g8 < 4 * WM; ++g8) {
                    int r = blk * BMr + g8 * 8 + lrow;
                    r = r < M ? r : M - 1;
                    const uint8_t *src = Ab + (long)r * g.lda * ES + ch * 16;
                    uint8_t *dst = slot + s2 * BMr * SLAB_BYTES + g8 * 8 * SLAB_BYTES;
                    if (ch < g.nch)
                        __builtin_amdgcn_global_load_lds((item_gas_ptr)src, (item_las_ptr)dst, 16, 0, 0);
                }
            }
        };
        // the bytes of the last chunk of a row that lie beyond K are whatever the caller's
        // buffer holds there: cleared in LDS before anybody reads the block
        auto fix_tail = [&](int blk) __attribute__((always_inline)) {
            if (tail_chunk >= 0 && lane < BMr) {
                uint8_t *p = sA0 + (blk % S) * abuf + (tail_chunk >> 3) * BMr * SLAB_BYTES + lane * SLAB_BYTES +
                             (((tail_chunk & 7) ^ (lane & 7)) * 16);
                i32x4 v = *reinterpret_cast<i32x4 *>(p);
                v = mask_chunk(v, kbytes - tail_chunk * 16);
                *reinterpret_cast<i32x4 *>(p) = v;
            }
        };
        if (RES) {
            for (int b2 = wave; b2 < g.nrb; b2 += 4) issue_block(b2);
        } else if (loader) {
            if (resident) {
                for (int b2 = 0; b2 < g.nrb; ++b2) issue_block(b2);
                item_wait_vmcnt(0);
                for (int b2 = 0; b2 < g.nrb; ++b2) fix_tail(b2);
            } else {
                for (int b2 = 0; b2 < S - 1; ++b2) issue_block(b2);
                item_wait_vmcnt((S - 2) * QL);                 // block 0 has arrived
                fix_tail(0);
            }
        }

        if (PROT && !loader) {
            for (int k = tid; k < 2 * nslab * KE; k += 256) a_lds[k] = 0u;     // a_lds and b_lds
            for (int n = tid; n < Nr; n += 256) ccobs[n] = 0u;
            for (int r = tid; r < Mr; r += 256) rcobs[r] = 0u;
            if (STO) for (int r = tid; r < Mr + Nr; r += 256) rcsto[r] = 0u;     // rcsto and ccsto
            if (tid < 16) misc[tid] = 0u;
        }
        float bmax = 0.f;                                        // max|B| seen by this thread

        // ---- B of this item into LDS, every position written (pads and rows past N with zeros)
        if (TRANSB) {
            const int cpr = nslab * 8;                           // chunk positions per row
            const int total = loader ? 0 : Nr * cpr;           // the loading wave takes no part
            for (int q0 = tid; q0 < total; q0 += 4 * 256) {
                i32x4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = q0 + 256 * u;
                    v[u] = i32x4{0, 0, 0, 0};
                    if (q < total) {
                        const int n = q / cpr, ch = q - n * cpr;
                        if (n < N && ch < g.nch) {
                            i32x4 x = *reinterpret_cast<const i32x4 *>(Bb + (long)n * g.ldb * ES + ch * 16);
                            if ((ch + 1) * 16 > kbytes) x = mask_chunk(x, kbytes - ch * 16);
                            v[u] = x;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = q0 + 256 * u;
                    if (q < total) {
                        const int n = q / cpr, ch = q - n * cpr;
                        *reinterpret_cast<i32x4 *>(sB + (size_t)(ch >> 3) * Nr * SLAB_BYTES + n * SLAB_BYTES +
                                                   (((ch & 7) ^ (n & 7)) * 16)) = v[u];
                    }
                }
            }
        } else {
            // B stored K x N: chunks run along n and are transposed on the way into LDS
            for (int q = tid; q < nslab * Nr * 8; q += NT)
                reinterpret_cast<i32x4 *>(sB)[q] = i32x4{0, 0, 0, 0};
            item_barrier();
            // A work item is KPT consecutive rows k of one chunk of columns: the KPT values of a
            // column make one 32-bit word of the transposed copy, so every LDS write is a word.
            constexpr int KPT = 4 / ES;
            const int cpr = (N + CE - 1) / CE;                   // chunks along n per row k
            const int total = loader ? 0 : ((K + KPT - 1) / KPT) * cpr;     // the loading wave takes no part
            for (int q0 = tid; q0 < total; q0 += 2 * 256) {
                i32x4 v[2][KPT];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int q = q0 + 256 * u;
                    const int kg = q / cpr, chn = q - kg * cpr;
#pragma unroll
                    for (int kk = 0; kk < KPT; ++kk) {
                        const int k = kg * KPT + kk;
                        v[u][kk] = i32x4{0, 0, 0, 0};
                        if (q < total && k < K)
                            v[u][kk] = *reinterpret_cast<const i32x4 *>(Bb + ((long)k * g.ldb + chn * CE) * ES);
                    }
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int q = q0 + 256 * u;
                    if (q < total) {
                        const int kg = q / cpr, chn = q - kg * cpr;
                        const int kb = kg * 4;                   // byte offset of the word along K
                        uint8_t *col = sB + (size_t)(kb >> 7) * Nr * SLAB_BYTES + (kb & 15);
                        const int kc = (kb >> 4) & 7;
                        acc_t part[KPT];                         // shares of b[k] = sum over n
#pragma unroll
                        for (int kk = 0; kk < KPT; ++kk) part[kk] = T::zero();
#pragma unroll
                        for (int e = 0; e < CE; ++e) {
                            const int n = chn * CE + e;
                            if (n < N) {
                                uint32_t word = 0;
#pragma unroll
                                for (int kk = 0; kk < KPT; ++kk) {
                                    if (PROT) {
                                        const acc_t x = T::elem(v[u][kk], e);
                                        part[kk] = add_t(part[kk], x);
                                        if (!T::IS_INT) bmax = fmaxf(bmax, fabsf((float)x));
                                    }
                                    if (ES == 2) {
                                        const uint32_t w = (uint32_t)v[u][kk][e >> 1];
                                        word |= ((e & 1) ? (w >> 16) : (w & 0xFFFFu)) << (16 * kk);
                                    } else {
                                        const uint32_t w = (uint32_t)v[u][kk][e >> 2];
                                        word |= ((w >> (8 * (e & 3))) & 0xFFu) << (8 * kk);
                                    }
                                }
                                *reinterpret_cast<uint32_t *>(col + n * SLAB_BYTES + ((kc ^ (n & 7)) * 16)) = word;
                            }
                        }
                        // a row of the stored B is a run of consecutive lanes: few lanes per word
                        if (PROT && !g.cached_b) {
#pragma unroll
                            for (int kk = 0; kk < KPT; ++kk) {
                                const int k = kg * KPT + kk;
                                if (k < K) {
                                    if constexpr (T::IS_INT) atomicAdd(reinterpret_cast<int *>(b_lds) + k, (int)part[kk]);
                                    else atomicAdd(reinterpret_cast<float *>(b_lds) + k, (float)part[kk]);
                                }
                            }
                        }
                    }
                }
            }
        }
        if (RES) {
            item_wait_vmcnt(0);                                  // this wave's blocks of A have arrived
            for (int b2 = wave; b2 < g.nrb; b2 += 4) fix_tail(b2);
        }
        item_barrier();

        // ---- b = B e and max|B| from the resident copy (or the cached encoding)
        if (PROT) {
            if (loader) {
                // nothing to do
            } else if (g.cached_b) {
                for (int k = tid; k < K; k += 256) b_lds[k] = g.b_sum[(long)bz * K + k];
            } else {
                // B stored N x K: column sums of the resident copy (stored K x N, the transposing
                // load above has already summed its rows)
                for (int s = 0; s < (TRANSB ? nslab : 0); ++s) {
                    acc_t cs[CE];
#pragma unroll
                    for (int q = 0; q < CE; ++q) cs[q] = T::zero();
                    for (int j = 0; j < NB; ++j) {
                        const i32x4 v = *reinterpret_cast<const i32x4 *>(
                            sB + (size_t)s * Nr * SLAB_BYTES + (rg + 32 * j) * SLAB_BYTES + ((c8 ^ (rg & 7)) * 16));
#pragma unroll
                        for (int q = 0; q < CE; ++q) {
                            const acc_t x = T::elem(v, q);
                            cs[q] = add_t(cs[q], x);
                            if (!T::IS_INT) bmax = fmaxf(bmax, fabsf((float)x));
                        }
                    }
#pragma unroll
                    for (int q = 0; q < CE; ++q) {
                        acc_t t = cs[q];
                        t = add_t(t, dpp_get<0x128>(t));          // lane ^ 8
                        t = add_xor16(t);
                        t = add_xor32(t);
                        cs[q] = t;
                    }
                    if (lane < 8) {
#pragma unroll
                        for (int q = 0; q < CE; ++q) {
                            if constexpr (T::IS_INT) atomicAdd(reinterpret_cast<int *>(b_lds) + s * KE + c8 * CE + q, (int)cs[q]);
                            else atomicAdd(reinterpret_cast<float *>(b_lds) + s * KE + c8 * CE + q, (float)cs[q]);
                        }
                    }
                }
                if (!T::IS_INT) {
                    bmax = wave_max(bmax);
                    if (lane == 0) misc[4 + wave] = __float_as_uint(bmax);
                }
            }
            item_barrier();
        }

        // ---- row blocks
        float amax = 0.f;
        // Column sums of A: chunk c8 of every slab, rows rg + 32 p of every row block.  int8: two
        // columns per register as 16-bit halves (a thread sees at most M / 32 <= 32 rows of a
        // column: |sum| <= 4096); dword d of a chunk gives csa[2 d] = columns 4 d + {0, 2} and
        // csa[2 d + 1] = columns 4 d + {1, 3}.
        typedef typename std::conditional<T::IS_INT, item_s16x2, float>::type csa_t;
        constexpr int NCSA = T::IS_INT ? CE / 2 : CE;
        csa_t csa[MAXS][NCSA];
#pragma unroll
        for (int s2 = 0; s2 < MAXS; ++s2)
#pragma unroll
            for (int q = 0; q < NCSA; ++q) {
                if constexpr (T::IS_INT) csa[s2][q] = item_s16x2{0, 0};
                else csa[s2][q] = 0.f;
            }
        // int8: the thread's sixteen values of b per slab as pairs of 16-bit halves, (b[4 d], b[4 d + 2])
        // and (b[4 d + 1], b[4 d + 3]), the order the pairs of A's bytes come in; they are the same for
        // every row block.  With |b| < 2^15 (N <= 255) that is bpk[slab].  Wider sums (|b| <= 128 N < 2^17)
        // are split, b = 256 hi + lo with 0 <= lo < 256, for a K of one slab: bpk[0] = hi, bpk[1] = lo.
        item_s16x2 bpk[T::IS_INT ? MAXS : 1][8];
        const bool b_split = T::IS_INT && !g.b16_ok && nslab == 1;
        if constexpr (T::IS_INT) {
            if (PROT && !loader && g.b16_ok) {
#pragma unroll
                for (int s2 = 0; s2 < MAXS; ++s2) {
                    const int sc = s2 < nslab ? s2 : nslab - 1;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const i32x4 w = *reinterpret_cast<const i32x4 *>(b_lds + sc * KE + c8 * CE + 4 * d);
                        bpk[s2][2 * d] = item_s16x2{(short)w[0], (short)w[2]};
                        bpk[s2][2 * d + 1] = item_s16x2{(short)w[1], (short)w[3]};
                    }
                }
            } else if (PROT && !loader && b_split) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const i32x4 w = *reinterpret_cast<const i32x4 *>(b_lds + c8 * CE + 4 * d);
                    bpk[0][2 * d] = item_s16x2{(short)(w[0] >> 8), (short)(w[2] >> 8)};
                    bpk[0][2 * d + 1] = item_s16x2{(short)(w[1] >> 8), (short)(w[3] >> 8)};
                    bpk[1][2 * d] = item_s16x2{(short)(w[0] & 255), (short)(w[2] & 255)};
                    bpk[1][2 * d + 1] = item_s16x2{(short)(w[1] & 255), (short)(w[3] & 255)};
                }
            }
        }
        acc_t cs[TPW][4];
        float cs_s[STO ? TPW : 1][4];            // column sums of the stored values
#pragma unroll
        for (int t = 0; t < TPW; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                cs[t][e] = T::zero();
                cs_s[STO ? t : 0][e] = 0.f;
            }

        // one row block, as the computing waves see it
        auto compute_block = [&](int rb) __attribute__((always_inline)) {
            const int m0 = rb * BMr;
            const uint8_t *sAc = sA0 + (rb % S) * abuf;
            if (PROT) {
                // The block's share of a = e^T A (kept in registers until the item ends), of the
                // row prediction A b and of max|A|: thread (c8, rg) reads chunk c8 of rows
                // rg + 32 p in every slab; a row's dot product is completed over its 8 lanes.
                // All of the thread's chunks are requested before the first is used (a slab past
                // the last reads the last again and is not used).
                auto a_pass = [&](auto mode_c) __attribute__((always_inline)) {
                    constexpr int MODE = decltype(mode_c)::value;   // 0: b as it is, 1: 16-bit pairs of b, 2: split b
                    constexpr bool B16 = MODE != 0;
                    acc_t dot[WM], dot_hi[WM];
#pragma unroll
                    for (int p = 0; p < WM; ++p) { dot[p] = T::zero(); dot_hi[p] = T::zero(); }
                    i32x4 xa[MAXS][WM];
#pragma unroll
                    for (int s2 = 0; s2 < MAXS; ++s2) {
                        const int sc = s2 < nslab ? s2 : nslab - 1;
#pragma unroll
                        for (int p = 0; p < WM; ++p)
                            xa[s2][p] = *reinterpret_cast<const i32x4 *>(sAc + sc * BMr * SLAB_BYTES +
                                                                         (rg + 32 * p) * SLAB_BYTES + ((c8 ^ (rg & 7)) * 16));
                    }
#pragma unroll
                    for (int s2 = 0; s2 < MAXS; ++s2) {
                        if (s2 < nslab) {
                            acc_t bv[CE];
                            if constexpr (!B16) {
#pragma unroll
                                for (int q4 = 0; q4 < CE / 4; ++q4) {
                                    const i32x4 w = *reinterpret_cast<const i32x4 *>(b_lds + s2 * KE + c8 * CE + 4 * q4);
#pragma unroll
                                    for (int e = 0; e < 4; ++e) bv[4 * q4 + e] = from_word<acc_t>((uint32_t)w[e]);
                                }
                            }
#pragma unroll
                            for (int p = 0; p < WM; ++p) {
                                i32x4 x4 = xa[s2][p];
                                if (m0 + rg + 32 * p >= M) x4 = i32x4{0, 0, 0, 0};
                                if constexpr (T::IS_INT) {
#pragma unroll
                                    for (int d = 0; d < 4; ++d) {
                                        const int wd = x4[d];
                                        const item_s16x2 w = item_s16x2{(short)(wd & 0xFFFF), (short)(wd >> 16)};
                                        const item_s16x2 ev = (w << 8) >> 8, od = w >> 8;   // bytes 0, 2 and 1, 3, sign-extended
                                        csa[s2][2 * d] += ev;
                                        csa[s2][2 * d + 1] += od;
                                        if constexpr (MODE == 1) {
                                            // the same pairs against pairs of b: two products per instruction
                                            dot[p] = __builtin_amdgcn_sdot2(ev, bpk[s2][2 * d], (int)dot[p], false);
                                            dot[p] = __builtin_amdgcn_sdot2(od, bpk[s2][2 * d + 1], (int)dot[p], false);
                                        }
                                        if constexpr (MODE == 2) {
                                            dot_hi[p] = __builtin_amdgcn_sdot2(ev, bpk[0][2 * d], (int)dot_hi[p], false);
                                            dot_hi[p] = __builtin_amdgcn_sdot2(od, bpk[0][2 * d + 1], (int)dot_hi[p], false);
                                            dot[p] = __builtin_amdgcn_sdot2(ev, bpk[1][2 * d], (int)dot[p], false);
                                            dot[p] = __builtin_amdgcn_sdot2(od, bpk[1][2 * d + 1], (int)dot[p], false);
                                        }
                                    }
                                }
                                if constexpr (!B16) {
#pragma unroll
                                    for (int q = 0; q < CE; ++q) {
                                        const acc_t x = T::elem(x4, q);
                                        if constexpr (!T::IS_INT) csa[s2][q] = csa[s2][q] + (float)x;
                                        if constexpr (T::IS_INT) {
                                            dot[p] = g.mul24_ok ? (acc_t)(__mul24((int)x, (int)bv[q]) + (int)dot[p])
                                                                : (acc_t)((uint32_t)x * (uint32_t)bv[q] + (uint32_t)dot[p]);
                                        } else {
                                            dot[p] = __builtin_fmaf((float)x, (float)bv[q], (float)dot[p]);
                                            amax = fmaxf(amax, fabsf((float)x));
                                        }
                                    }
                                }
                            }
                        }
                    }
#pragma unroll
                    for (int p = 0; p < WM; ++p) {
                        if constexpr (MODE == 2) dot[p] = (acc_t)((uint32_t)dot_hi[p] * 256u + (uint32_t)dot[p]);
                        const acc_t d = row8_sum(dot[p]);
                        if (c8 == p) rcpred[m0 + rg + 32 * p] = as_word(d);
                    }
                };
                if constexpr (T::IS_INT) {
                    if (g.b16_ok) a_pass(std::integral_constant<int, 1>{});
                    else if (b_split) a_pass(std::integral_constant<int, 2>{});
                    else a_pass(std::integral_constant<int, 0>{});
                } else {
                    a_pass(std::integral_constant<int, 0>{});
                }
            }

            accv_t acc[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[t][i] = T::zero();
            const bool mact = (m0 + wm * 32) < M;
            if (mact && TPW <= 2) {
                // narrow tiles: with one or two MFMAs per step of K, the LDS latency of a step's
                // fragments is several MFMAs long, so the reads run FD - 1 = 3 steps ahead of the
                // MFMAs (a slab is four steps).  A column block past the last one reads the last one again (its
                // products are never used).
                constexpr int FD = 4;
                const uint8_t *fa = sAc + (wm * 32 + l32) * SLAB_BYTES;
                const uint8_t *fb[TPW];
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    int nb = t * WN + wn;
                    nb = nb < NB ? nb : NB - 1;
                    fb[t] = sB + (nb * 32 + l32) * SLAB_BYTES;
                }
                const int bslab = Nr * SLAB_BYTES, aslab = BMr * SLAB_BYTES;
                i32x4 af[FD], bf[FD][TPW];
                auto frag_load = [&](int k1, auto slot_c) __attribute__((always_inline)) {
                    constexpr int slot = decltype(slot_c)::value;
                    const int s1 = k1 >> 2, sw = ((2 * (k1 & 3) + lh) ^ (lane & 7)) * 16;
                    af[slot] = *reinterpret_cast<const i32x4 *>(fa + s1 * aslab + sw);
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
                        bf[slot][t] = *reinterpret_cast<const i32x4 *>(fb[t] + (size_t)s1 * bslab + sw);
                };
                // Whole slabs, four steps each, without conditions (the steps past K multiply the
                // zero padding of the slab): straight-line code lets the waits count exactly.
                static_for<0, FD - 1>([&](auto d_c) { frag_load(decltype(d_c)::value, d_c); });
                for (int s1 = 0; s1 < nslab - 1; ++s1) {
                    static_for<0, FD>([&](auto h_c) {
                        constexpr int h = decltype(h_c)::value;
                        frag_load(4 * s1 + h + FD - 1, std::integral_constant<int, (h + FD - 1) % FD>{});
#pragma unroll
                        for (int t = 0; t < TPW; ++t) acc[t] = T::mfma(bf[h][t], af[h], acc[t]);
                    });
                }
                frag_load(4 * (nslab - 1) + FD - 1, std::integral_constant<int, FD - 1>{});
                static_for<0, FD>([&](auto h_c) {
                    constexpr int h = decltype(h_c)::value;
#pragma unroll
                    for (int t = 0; t < TPW; ++t) acc[t] = T::mfma(bf[h][t], af[h], acc[t]);
                });
            } else if (mact) {
                for (int ks = 0; ks < g.ksteps; ++ks) {
                    const int s = ks >> 2, s4 = ks & 3;
                    const int sw = ((2 * s4 + lh) ^ (lane & 7)) * 16;
                    const i32x4 af = *reinterpret_cast<const i32x4 *>(sAc + s * BMr * SLAB_BYTES +
                                                                      (wm * 32 + l32) * SLAB_BYTES + sw);
#pragma unroll
                    for (int t = 0; t < TPW; ++t) {
                        const int nb = t * WN + wn;
                        if (nb < NB) {
                            const i32x4 bf = *reinterpret_cast<const i32x4 *>(
                                sB + (size_t)s * Nr * SLAB_BYTES + (nb * 32 + l32) * SLAB_BYTES + sw);
                            acc[t] = T::mfma(bf, af, acc[t]);
                        }
                    }
                }
            }

            // ---- epilogue of the row block: block by block through the wave's LDS stage.
            // Lane l holds row l & 31 of a block and in register i column 8 (i >> 2) + 4 (l >> 5)
            // + (i & 3); read back, lane l has four consecutive columns 4 (l & 7) .. of row
            // 8 p + (l >> 3): eight lanes cover a 32-column row segment.
            acc_t rsum[4] = {T::zero(), T::zero(), T::zero(), T::zero()};
            float rsum_s[4] = {0.f, 0.f, 0.f, 0.f};
            const int row0 = m0 + wm * 32 + (lane >> 3);             // this lane's row of pass 0; pass p: + 8 p
            const long rowstep = 8 * g.ldc * OS;
            uint8_t *dst_row0 = Cb + ((long)row0 * g.ldc + 4 * (lane & 7)) * OS;
            const bool inj_blk = PROT && bz == g.inj_b && g.inj_row >= m0 && g.inj_row < m0 + BMr;
            static_for<0, TPW>([&](auto t_c) {
                constexpr int t = decltype(t_c)::value;
                const int nb = t * WN + wn;
                if (mact && nb < NB) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<i32x4 *>(stage + (l32 * ITEM_STAGE_ROW + 8 * q + 4 * lh) * 4) =
                            i32x4{(int)as_word(acc[t][4 * q]), (int)as_word(acc[t][4 * q + 1]),
                                  (int)as_word(acc[t][4 * q + 2]), (int)as_word(acc[t][4 * q + 3])};
                    wave_sync();
                    i32x4 w4[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p)
                        w4[p] = *reinterpret_cast<const i32x4 *>(
                            stage + ((8 * p + (lane >> 3)) * ITEM_STAGE_ROW + 4 * (lane & 7)) * 4);
                    wave_sync();                                  // the stage is free for the next block
                    const int gc = nb * 32 + 4 * (lane & 7);
                    uint8_t *dst_blk = dst_row0 + (long)nb * 32 * OS;
                    const bool cfull = gc + 4 <= N;
                    if (inj_blk) {
#pragma unroll
                        for (int p = 0; p < 4; ++p)
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (row0 + 8 * p == g.inj_row && g.inj_col == gc + e) w4[p][e] ^= (int)(1u << g.inj_bit);
                    }
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const bool rv = row0 + 8 * p < M;          // rows past M hold a copy of the last row
                        acc_t v[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = from_word<acc_t>((uint32_t)w4[p][e]);
                        if (PROT) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) cs[t][e] = add_t(cs[t][e], rv ? v[e] : T::zero());
                            rsum[p] = add_t(rsum[p], add_t(add_t(v[0], v[1]), add_t(v[2], v[3])));
                        }
                        // Plain stores: the row segments of neighbouring blocks complete each other's
                        // cache lines (rows of C are not line-aligned), which the L2 merges;
                        // streaming stores sent the partial lines to memory one by one and ran
                        // three to five times slower here.
                        uint8_t *dst = dst_blk + p * rowstep;
                        if constexpr (T::IS_INT) {
                            if (rv && cfull) {
                                *reinterpret_cast<i32x4 *>(dst) = w4[p];
                            } else if (rv) {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (gc + e < N) reinterpret_cast<int *>(dst)[e] = w4[p][e];
                            }
                        } else {
                            const uint32_t lo = pack2<DT>((float)v[0], (float)v[1]);
                            const uint32_t hi = pack2<DT>((float)v[2], (float)v[3]);
                            if constexpr (STO) {
                                float sv[4];
                                if constexpr (DT == DT_BF16) {
                                    sv[0] = __uint_as_float(lo << 16); sv[1] = __uint_as_float(lo & 0xFFFF0000u);
                                    sv[2] = __uint_as_float(hi << 16); sv[3] = __uint_as_float(hi & 0xFFFF0000u);
                                } else {
                                    sv[0] = f16_bits_to_f32(lo & 0xFFFFu); sv[1] = f16_bits_to_f32(lo >> 16);
                                    sv[2] = f16_bits_to_f32(hi & 0xFFFFu); sv[3] = f16_bits_to_f32(hi >> 16);
                                }
#pragma unroll
                                for (int e = 0; e < 4; ++e) cs_s[t][e] += rv ? sv[e] : 0.f;
                                rsum_s[p] += (sv[0] + sv[1]) + (sv[2] + sv[3]);
                            }
                            if (rv && cfull) {
                                typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
                                *reinterpret_cast<u32x2 *>(dst) = u32x2{lo, hi};
                            } else if (rv) {
                                uint16_t *d16 = reinterpret_cast<uint16_t *>(dst);
                                if (gc + 0 < N) d16[0] = (uint16_t)(lo & 0xFFFFu);
                                if (gc + 1 < N) d16[1] = (uint16_t)(lo >> 16);
                                if (gc + 2 < N) d16[2] = (uint16_t)(hi & 0xFFFFu);
                                if (gc + 3 < N) d16[3] = (uint16_t)(hi >> 16);
                            }
                        }
                    }
                }
            });
            if (PROT) {
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    // the waves that share these rows add their parts (distinct words per lane)
                    const acc_t r = row8_sum(rsum[p]);
                    // (the add as the instruction itself: through atomicAdd the compiler, which
                    // cannot tell these words from the targets of the direct-to-LDS loads, makes the
                    // wave wait for every store of C it has in flight before each add)
                    if ((lane & 7) == 0 && mact) lds_add_word(rcobs + m0 + wm * 32 + 8 * p + (lane >> 3), r);
                    if constexpr (STO) {
                        const float rs = row8_sum(rsum_s[p]);
                        if ((lane & 7) == 0 && mact) lds_add_word(rcsto + m0 + wm * 32 + 8 * p + (lane >> 3), rs);
                    }
                }
            }
        };
        for (int rb = 0; rb < g.nrb; ++rb) {
            if (!loader) {
                compute_block(rb);
            } else if (!resident) {
                // S - 1 blocks ahead; then block rb + 1 must be in place behind this barrier
                issue_block(rb + S - 1);
                item_wait_vmcnt((S - 2) * QL);
                fix_tail(rb + 1);
            }
            if (!resident) item_barrier();
        }
        item_barrier();

        if (loader) item_wait_vmcnt(0);                         // the blocks fetched past the end

        // ---- the item's checks (computing waves)
        // the waves' partial column sums of C and of A meet in LDS
        auto reduce_sums = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const int nb = t * WN + wn;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc_t v = cs[t][e];
                    v = add_t(v, dpp_get<0x128>(v));              // lane ^ 8
                    v = add_xor16(v);
                    v = add_xor32(v);
                    if (lane < 8 && nb < NB) {
                        uint32_t *dst = ccobs + nb * 32 + 4 * lane + e;
                        if (WM == 1) *dst = as_word(v);
                        else lds_add_word(dst, v);
                    }
                    if constexpr (STO) {
                        float vs = cs_s[t][e];
                        vs = add_t(vs, dpp_get<0x128>(vs));       // lane ^ 8
                        vs = add_xor16(vs);
                        vs = add_xor32(vs);
                        if (lane < 8 && nb < NB) lds_add_word(ccsto + nb * 32 + 4 * lane + e, vs);
                    }
                }
            }
            // a = e^T A: over the eight row groups of the wave in registers (int8: still as pairs
            // of 16-bit halves: 256 rows of bytes fit), then one copy per wave in the wave's
            // staging area, which the epilogues are done with; sum_waves adds the four copies
            uint32_t *mine = reinterpret_cast<uint32_t *>(stage);
#pragma unroll
            for (int s2 = 0; s2 < MAXS; ++s2) {
                i32x4 out[2];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if constexpr (T::IS_INT) {
                        int w = item_word(csa[s2][j]);
                        w = item_word(item_pair(w) + item_pair(dpp_get<0x128>(w)));          // lane ^ 8
                        auto p16 = __builtin_amdgcn_permlane16_swap((unsigned)w, (unsigned)w, false, false);
                        w = item_word(item_pair((int)p16[0]) + item_pair((int)p16[1]));      // lane ^ 16
                        auto p32 = __builtin_amdgcn_permlane32_swap((unsigned)w, (unsigned)w, false, false);
                        w = item_word(item_pair((int)p32[0]) + item_pair((int)p32[1]));      // lane ^ 32
                        out[j >> 2][j & 3] = w;
                    } else {
                        float v = csa[s2][j];
                        v = add_t(v, dpp_get<0x128>(v));              // lane ^ 8
                        v = add_xor16(v);
                        v = add_xor32(v);
                        out[j >> 2][j & 3] = (int)__float_as_uint(v);
                    }
                }
                if (lane < 8 && s2 < nslab) {
                    i32x4 *dst = reinterpret_cast<i32x4 *>(mine + (s2 * 8 + lane) * 8);
                    dst[0] = out[0];
                    dst[1] = out[1];
                }
            }
            if (!T::IS_INT) {
                const float m = wave_max(amax);
                if (lane == 0) misc[wave] = __float_as_uint(m);
            }
        };
        // a[k] from the four waves' copies (int8: column 4 d + e of a chunk sits in half (e >> 1) of
        // word 2 d + (e & 1))
        auto sum_waves = [&]() __attribute__((always_inline)) {
            for (int k = tid; k < nslab * KE; k += 256) {
                const int s2 = k / KE, c = (k % KE) / CE, q = k % CE;
                acc_t t = T::zero();
#pragma unroll
                for (int w2 = 0; w2 < 4; ++w2) {
                    const uint32_t *copy = reinterpret_cast<const uint32_t *>(sA0 + S * abuf + w2 * ITEM_STAGE_WAVE) +
                                           (s2 * 8 + c) * 8;
                    if constexpr (T::IS_INT) {
                        const uint32_t wd = copy[2 * (q >> 2) + (q & 1)];
                        t += (int)(short)(((q >> 1) & 1) ? (wd >> 16) : (wd & 0xFFFFu));
                    } else {
                        t += __uint_as_float(copy[q]);
                    }
                }
                a_lds[k] = as_word(t);
            }
        };
        // a B from the resident B against the column sums; row sums against A b; vectors out
        auto check_item = [&](float tol) __attribute__((always_inline)) {
            // columns: prediction a B from the resident B; LPC lanes share a column (four where
            // there are at most 64 columns, so that all 256 threads take part)
            constexpr int LPC = WM == 2 ? 4 : 1;
            for (int n0 = 0; n0 < N; n0 += 256 / LPC) {
                const int n = n0 + tid / LPC, part = tid % LPC;
                bool fl = false;
                acc_t dot = T::zero();
                if (n < N) {
                    for (int ch = part; ch < g.nch; ch += LPC) {
                        const i32x4 v = *reinterpret_cast<const i32x4 *>(
                            sB + (size_t)(ch >> 3) * Nr * SLAB_BYTES + n * SLAB_BYTES + (((ch & 7) ^ (n & 7)) * 16));
                        const i32x4 *ap = reinterpret_cast<const i32x4 *>(a_lds + ch * CE);
#pragma unroll
                        for (int q4 = 0; q4 < CE / 4; ++q4) {
                            const i32x4 aw = ap[q4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                // int8: |a| <= 128 M < 2^23 here (M <= 1024): 24-bit multiplies are exact
                                if constexpr (T::IS_INT) dot = __mul24((int)T::elem(v, 4 * q4 + e), aw[e]) + dot;
                                else dot = add_t(dot, mul_t(T::elem(v, 4 * q4 + e), from_word<acc_t>((uint32_t)aw[e])));
                            }
                        }
                    }
                }
                if (LPC == 4) {
                    dot = add_t(dot, dpp_get<0xB1>(dot));         // lane ^ 1
                    dot = add_t(dot, dpp_get<0x4E>(dot));         // lane ^ 2
                }
                if (n < N && part == 0) {
                    const long o = (long)bz * N + n;
                    const uint32_t obs = ccobs[n];
                    g.cc_pred[o] = as_word(dot);
                    g.cc_obs[o] = obs;
                    if (STO) g.cc_sto[o] = ccsto[n];
                    fl = mismatch<T::IS_INT>(obs, as_word(dot), g.tau_override_cols > 0.f ? g.tau_override_cols : tol);
                    g.col_flag[o] = fl ? 1 : 0;
                }
                nc_w += __popcll(__ballot(fl));
            }
            for (int r0 = 0; r0 < M; r0 += 256) {
                const int r = r0 + tid;
                bool fl = false;
                if (r < M) {
                    const long o = (long)bz * M + r;
                    const uint32_t obs = rcobs[r], pred = rcpred[r];
                    g.rc_obs[o] = obs;
                    g.rc_pred[o] = pred;
                    if (STO) g.rc_sto[o] = rcsto[r];
                    fl = mismatch<T::IS_INT>(obs, pred, tol);
                    g.row_flag[o] = fl ? 1 : 0;
                }
                nr_w += __popcll(__ballot(fl));
            }
            acc_t sp = T::zero();
            for (int k = tid; k < K; k += 256) {
                const uint32_t aw = a_lds[k], bw = b_lds[k];
                g.a_sum[(long)bz * K + k] = aw;
                if (!g.cached_b) g.b_sum[(long)bz * K + k] = bw;
                sp = add_t(sp, mul_t(from_word<acc_t>(aw), from_word<acc_t>(bw)));
            }
            sp = wave_sum(sp);
            if (lane == 0) misc[8 + wave] = as_word(sp);
        };
        if (PROT) {
            if (!loader) reduce_sums();
            item_barrier();
            if (!loader) sum_waves();
            item_barrier();
            float tol = 0.f, ma = 0.f, mb = 0.f;
            if (!T::IS_INT) {
                ma = fmaxf(fmaxf(__uint_as_float(misc[0]), __uint_as_float(misc[1])),
                           fmaxf(__uint_as_float(misc[2]), __uint_as_float(misc[3])));
                mb = g.cached_b ? __uint_as_float(g.b_max[bz])
                                : fmaxf(fmaxf(__uint_as_float(misc[4]), __uint_as_float(misc[5])),
                                        fmaxf(__uint_as_float(misc[6]), __uint_as_float(misc[7])));
                tol = g.tau_override > 0.f ? g.tau_override : (1e-3f * (float)K) * ma * mb;
            }
            if (!loader) check_item(tol);
            item_barrier();
            if (tid == 0) {
                g.s_pred[bz] = as_word(add_t(add_t(from_word<acc_t>(misc[8]), from_word<acc_t>(misc[9])),
                                             add_t(from_word<acc_t>(misc[10]), from_word<acc_t>(misc[11]))));
                if (!T::IS_INT) {
                    g.maxabs[(long)bz * 2] = ma;
                    g.maxabs[(long)bz * 2 + 1] = mb;
                    g.tau[bz] = tol;
                    g.a_max[bz] = __float_as_uint(ma);
                    if (!g.cached_b) g.b_max[bz] = __float_as_uint(mb);
                }
            }
        }
        item_barrier();                                        // LDS is reused by the next item
    }

    if (PROT) {
        // flagged rows / columns of this workgroup, then its ticket (in two levels: atomics on
        // one word are served one after the other); the last workgroup writes counts and status
        if (lane == 0 && !loader) { misc[16 + wave] = nr_w; misc[20 + wave] = nc_w; }
        item_barrier();
        if (tid == 0) {
            const unsigned nr = misc[16] + misc[17] + misc[18] + misc[19];
            const unsigned nc = misc[20] + misc[21] + misc[22] + misc[23];
            if (nr | nc) {
                // rare: the counts must have arrived before this workgroup's ticket does
                unsigned o1 = 0, o2 = 0;
                if (nr) o1 = atomicAdd(g.ticket + 1, nr);
                if (nc) o2 = atomicAdd(g.ticket + 2, nc);
                asm volatile("s_waitcnt vmcnt(0)" :: "v"(o1), "v"(o2) : "memory");
            }
            const unsigned grp = blockIdx.x / ITEM_GROUP, ngrp = (gridDim.x + ITEM_GROUP - 1) / ITEM_GROUP;
            const unsigned gsize = min((unsigned)ITEM_GROUP, gridDim.x - grp * ITEM_GROUP);
            bool last = false;
            if (atomicAdd(g.group_ticket + grp, 1u) == gsize - 1) {
                atomicExch(g.group_ticket + grp, 0u);
                last = atomicAdd(g.ticket, 1u) == ngrp - 1;
            }
            if (last) {
                const uint32_t r = atomicExch(g.ticket + 1, 0u), c = atomicExch(g.ticket + 2, 0u);
                atomicExch(g.ticket, 0u);
                g.counts[0] = r;
                g.counts[1] = c;
                g.counts[2] = status_of(r, c);
                g.counts[3] = 0u;
                g.counts[4] = status_of(r, c);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
static void item_config(int N, int *wm, int *tpw)
{
    if (N <= 64) { *wm = 2; *tpw = 1; }
    else if (N <= 256) { *wm = 1; *tpw = 2; }
    else { *wm = 1; *tpw = 5; }
}

bool gemm_item_eligible(int dt, const Shape &s, bool stored_sums)
{
    const int es = elem_size(dt);
    const bool sto = stored_sums && dt != DT_I8;
    if (s.batch < ITEM_MIN_BATCH) return false;
    if (s.N > 640 || s.M > ITEM_MAX_M) return false;
    if ((long)s.K * es > ITEM_MAX_SLABS * SLAB_BYTES) return false;
    int wm, tpw;
    item_config(s.N, &wm, &tpw);
    if (sto && tpw > 2) return false;                      // wide tiles have no registers to spare for them
    if (((long)s.K * es + SLAB_BYTES - 1) / SLAB_BYTES > item_max_slabs(wm, tpw)) return false;
    return item_stages(dt, wm, s.M, s.N, s.K, sto) > 0;
}

template <int DT, int WM, int TPW, bool PROT, bool TRANSB, bool RES, bool STO>
static hipError_t launch_item_sto(const ItemArgs &g, size_t smem, hipStream_t st)
{
    auto kern = gemm_item_kernel<DT, WM, TPW, PROT, TRANSB, RES, STO>;
    hipError_t e = ensure_max_lds(reinterpret_cast<const void *>(kern), ITEM_LDS_LIMIT);
    if (e != hipSuccess) return e;
    const unsigned blocks = (unsigned)(g.batch < ITEM_MAX_BLOCKS ? g.batch : ITEM_MAX_BLOCKS);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(RES ? 256 : ITEM_THREADS), smem, st, g);
    return hipGetLastError();
}

template <int DT, int WM, int TPW, bool PROT, bool TRANSB, bool RES>
static hipError_t launch_item_res(const ItemArgs &g, size_t smem, hipStream_t st)
{
    if constexpr (PROT && DT != DT_I8 && TPW <= 2) {
        if (g.cc_sto) return launch_item_sto<DT, WM, TPW, PROT, TRANSB, RES, true>(g, smem, st);
    }
    return launch_item_sto<DT, WM, TPW, PROT, TRANSB, RES, false>(g, smem, st);
}

template <int DT, int WM, int TPW, bool PROT, bool TRANSB>
static hipError_t launch_item_one(const ItemArgs &g, size_t smem, hipStream_t st)
{
    if constexpr (TPW <= 2) {
        if (g.stages >= g.nrb) return launch_item_res<DT, WM, TPW, PROT, TRANSB, true>(g, smem, st);
    }
    return launch_item_res<DT, WM, TPW, PROT, TRANSB, false>(g, smem, st);
}

template <int DT, int WM, int TPW>
static hipError_t launch_item_cfg(bool protect, bool transB, const ItemArgs &g, size_t smem, hipStream_t st)
{
    if (protect) return transB ? launch_item_one<DT, WM, TPW, true, true>(g, smem, st)
                               : launch_item_one<DT, WM, TPW, true, false>(g, smem, st);
    return transB ? launch_item_one<DT, WM, TPW, false, true>(g, smem, st)
                  : launch_item_one<DT, WM, TPW, false, false>(g, smem, st);
}

template <int DT>
static hipError_t launch_item_dt(int wm, int tpw, bool protect, bool transB, const ItemArgs &g, size_t smem,
                                 hipStream_t st)
{
    if (wm == 2) return launch_item_cfg<DT, 2, 1>(protect, transB, g, smem, st);
    if (tpw == 2) return launch_item_cfg<DT, 1, 2>(protect, transB, g, smem, st);
    return launch_item_cfg<DT, 1, 5>(protect, transB, g, smem, st);
}

hipError_t launch_gemm_item(int dt, bool protect, bool cached_b, bool stored_sums, const void *A, const void *B, void *C,
                            const Shape &s, const Workspace &w, const Verdict *v, const InjectArm &arm,
                            hipStream_t st)
{
    const bool sto = protect && stored_sums && dt != DT_I8;
    if (!gemm_item_eligible(dt, s, sto)) return hipErrorInvalidValue;
    if (protect && v == nullptr) return hipErrorInvalidValue;
    const int es = elem_size(dt);
    int wm, tpw;
    item_config(s.N, &wm, &tpw);
    ItemArgs g;
    g.A = (const uint8_t *)A; g.B = (const uint8_t *)B; g.C = (uint8_t *)C;
    g.M = s.M; g.N = s.N; g.K = s.K; g.batch = s.batch;
    g.lda = s.lda; g.ldb = s.ldb; g.ldc = s.ldc; g.sA = s.sA; g.sB = s.sB; g.sC = s.sC;
    g.nslab = (s.K * es + SLAB_BYTES - 1) / SLAB_BYTES;
    g.nch = (s.K * es + 15) / 16;
    g.ksteps = (s.K * es + 31) / 32;
    g.NB = (s.N + 31) / 32;
    g.nrb = (s.M + 32 * wm - 1) / (32 * wm);
    g.stages = item_stages(dt, wm, s.M, s.N, s.K, sto);
    g.inj_b = arm.batch; g.inj_row = arm.row; g.inj_col = arm.col; g.inj_bit = arm.bit;
    g.mul24_ok = s.N < 65536 ? 1 : 0;
    g.b16_ok = s.N <= 255 ? 1 : 0;
    g.cached_b = cached_b ? 1 : 0;
    g.cc_obs = w.cc_obs; g.rc_obs = w.rc_obs; g.rc_pred = w.rc_pred; g.a_sum = w.a_sum; g.a_max = w.a_max;
    g.b_sum = w.b_sum; g.b_max = w.b_max; g.cc_pred = w.cc_pred; g.s_pred = w.s_pred;
    g.cc_sto = sto ? w.cc_sto : nullptr; g.rc_sto = sto ? w.rc_sto : nullptr;
    g.maxabs = w.maxabs; g.tau = w.tau;
    g.tau_override = v ? v->tau_override : 0.f;
    g.tau_override_cols = v ? v->tau_override_cols : 0.f;
    g.row_flag = v ? v->row_flag : nullptr; g.col_flag = v ? v->col_flag : nullptr;
    g.counts = v ? v->counts : nullptr;
    g.ticket = w.cmp_ticket; g.group_ticket = w.cmp_ticket + 4;
    const size_t smem = item_lds_bytes(dt, wm, g.stages, s.M, s.N, s.K, sto);
    switch (dt) {
    case DT_I8:   return launch_item_dt<DT_I8>(wm, tpw, protect, s.transB != 0, g, smem, st);
    case DT_BF16: return launch_item_dt<DT_BF16>(wm, tpw, protect, s.transB != 0, g, smem, st);
    case DT_F16:  return launch_item_dt<DT_F16>(wm, tpw, protect, s.transB != 0, g, smem, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace abft
