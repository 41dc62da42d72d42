// C-ABI of libabft: context, argument validation, workspace carving, launch order.
// Every hot call only enqueues kernels on the caller's stream.
#include <hip/hip_runtime.h>
#include <mutex>
#include <new>
#include <vector>
#include <string.h>

#include "../../include/abft.h"
#include "abft_internal.h"

using namespace abft;

struct abft_ctx {
    abft_config cfg;
    // device pools (32-bit words unless noted)
    uint32_t *pool_depth;   // two slots of (max_depth + max_batch) words: b = B e, then max|B| per batch item
    size_t bslot_words;     // words per slot
    int bslot;              // slot that holds the b in use
    bool bclean[2];         // slot is all zero
    uint32_t *pool_batch;   // per-batch scalars
    uint32_t *pool_cols;    // cc_pred
    uint32_t *pool_obs;     // two regions of cc_obs | rc_obs | rc_pred | a_sum | a_max | cc_sto | rc_sto:
                            // protected GEMMs alternate between them; each must be clean before use
    size_t region_words;    // words per region
    int cur;                // region of the last protected GEMM
    size_t dirty[2];        // leading words of each region that may be non-zero
    uint32_t *pool_vobs;    // two regions of cc_vobs | rc_vobs, used alternately like pool_obs
    size_t vregion_words;
    int vcur;
    size_t vdirty[2];
    int32_t  *fix_tiles;
    uint32_t *small;        // fix_count[4], cmp_ticket[4], group tickets of the finish kernel [64]
    InjectArm arm;
    int last_hip;
    // what the context currently holds
    bool b_valid, pred_valid, sto_valid, vobs_valid;
    bool is_static;         // the context of abft_gemm_static: its pools are not allocations
    bool graph_mode;        // a call of this context has been captured into a graph (sticky): see in_graph_mode
    bool vobs_captured;     // ... and they were formed by a call enqueued under capture
    const void *vobs_C;     // the stored C the re-summed vectors belong to (with its ldc and batch stride)
    int64_t vobs_ldc, vobs_strideC;
    bool list_dirty;        // the tile list's counters may be non-zero (a correction failed half way)
    int b_dt, pred_dt;
    const void *given_a, *given_amax;   // abft_supply_a: a = e^T A and max|A| for the next call with ABFT_A_CHECKSUM_GIVEN
    hipEvent_t done_event;              // abft_gemm_done_event: recorded behind every GEMM kernel (null: none)
    const void *pred_bias;  // layer bias of the GEMM the predictions belong to (abft_correct adds it to recomputed tiles)
    abft_shape b_shape, pred_shape;
    // optional kernel timing (abft_profile_begin / _end)
    hipEvent_t *prof_ev;    // 4 events per recorded call
    int prof_cap, prof_n;
};

static const int BATCH_WORDS = 2 /*maxabs*/ + 1 /*tau*/ + 1 /*s_pred*/;

static int fail_hip(abft_ctx *c, hipError_t e)
{
    if (c) c->last_hip = (int)e;
    return ABFT_EHIP;
}

static int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

extern "C" int abft_version(void) { return 100; }

extern "C" const char *abft_strerror(int code)
{
    switch (code) {
    case ABFT_OK: return "ok";
    case ABFT_EINVAL: return "invalid argument";
    case ABFT_EALIGN: return "pointer, leading dimension or stride not a multiple of 16 bytes";
    case ABFT_ESHAPE: return "bad shape";
    case ABFT_EWORKSPACE: return "shape exceeds the context's workspace";
    case ABFT_EHIP: return "HIP runtime error";
    case ABFT_ESTATE: return "required state missing in the context";
    default: return "unknown error";
    }
}

extern "C" int abft_last_hip_error(const abft_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

// The device pools of a context, in 32-bit words, for a context that serves max_rows / max_cols /
// max_depth (already rounded, see abft_create) / max_batch.
constexpr int N_POOLS = 7;
static constexpr size_t pool_total_words(size_t R, size_t Cn, size_t D, size_t Bt)
{
    return 2 * (D + Bt) + Bt * BATCH_WORDS + Cn + 2 * (2 * Cn + 3 * R + D + 2 * Bt) + 2 * (R + Cn) +
           (size_t)MAX_FIX_TILES * 3 + (8 + 64);
}
static void pool_words(int64_t max_rows, int64_t max_cols, int64_t max_depth, int64_t max_batch, size_t words[N_POOLS])
{
    const size_t D = (size_t)max_depth, R = (size_t)max_rows, Cn = (size_t)max_cols, Bt = (size_t)max_batch;
    words[0] = 2 * (D + Bt);                       // pool_depth
    words[1] = Bt * BATCH_WORDS;                   // pool_batch
    words[2] = Cn;                                 // pool_cols
    words[3] = 2 * (2 * Cn + 3 * R + D + 2 * Bt);  // pool_obs
    words[4] = 2 * (R + Cn);                       // pool_vobs
    words[5] = (size_t)MAX_FIX_TILES * 3;          // fix_tiles
    words[6] = 8 + 64;                             // small
}
static void pool_slots(abft_ctx *c, void **slot[N_POOLS])
{
    slot[0] = (void **)&c->pool_depth; slot[1] = (void **)&c->pool_batch; slot[2] = (void **)&c->pool_cols;
    slot[3] = (void **)&c->pool_obs;   slot[4] = (void **)&c->pool_vobs;  slot[5] = (void **)&c->fix_tiles;
    slot[6] = (void **)&c->small;
}
// Host-side bookkeeping of a context whose pools are all zero.
static void start_clean(abft_ctx *c)
{
    const size_t D = (size_t)c->cfg.max_depth, R = (size_t)c->cfg.max_rows, Cn = (size_t)c->cfg.max_cols,
                 Bt = (size_t)c->cfg.max_batch;
    c->region_words = 2 * Cn + 3 * R + D + 2 * Bt;
    c->cur = 0;
    c->dirty[0] = c->dirty[1] = 0;
    c->vregion_words = R + Cn;
    c->vcur = 0;
    c->vdirty[0] = c->vdirty[1] = 0;
    c->bslot_words = D + Bt;
    c->bslot = 0;
    c->bclean[0] = c->bclean[1] = true;
}

extern "C" int abft_create(abft_ctx **out, const abft_config *cfg)
{
    if (!out || !cfg) return ABFT_EINVAL;
    *out = nullptr;
    if (cfg->max_rows < 1 || cfg->max_cols < 1 || cfg->max_depth < 1 || cfg->max_batch < 1) return ABFT_ESHAPE;
    abft_ctx *c = new (std::nothrow) abft_ctx;
    if (!c) return ABFT_EINVAL;
    memset(c, 0, sizeof(*c));
    c->cfg = *cfg;
    c->cfg.max_depth = round_up(cfg->max_depth, SLAB_BYTES) + (int64_t)SLAB_BYTES * cfg->max_batch;
    c->arm.batch = -1;
    hipError_t e = hipSetDevice(cfg->device);
    if (e != hipSuccess) { int r = fail_hip(c, e); delete c; return r; }
    size_t words[N_POOLS];
    pool_words(c->cfg.max_rows, c->cfg.max_cols, c->cfg.max_depth, c->cfg.max_batch, words);
    void **slot[N_POOLS];
    pool_slots(c, slot);
    for (int i = 0; i < N_POOLS; ++i) {
        e = hipMalloc(slot[i], words[i] * 4);
        if (e == hipSuccess) e = hipMemset(*slot[i], 0, words[i] * 4);
        if (e != hipSuccess) {
            int r = fail_hip(c, e);
            abft_destroy(c);
            return r;
        }
    }
    e = hipDeviceSynchronize();
    if (e != hipSuccess) { int r = fail_hip(c, e); abft_destroy(c); return r; }
    start_clean(c);
    *out = c;
    return ABFT_OK;
}

static void prof_free(abft_ctx *c);

extern "C" int abft_destroy(abft_ctx *c)
{
    if (!c || c->is_static) return ABFT_EINVAL;
    prof_free(c);
    void *ptrs[] = {c->pool_depth, c->pool_batch, c->pool_cols, c->pool_obs, c->pool_vobs, c->fix_tiles, c->small};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete c;
    return ABFT_OK;
}

// ------------------------------------------------------------------------------------------
static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// need: 1 = A, 2 = B, 4 = C
static int check_shape(const abft_ctx *c, int dt, const abft_shape *s, int need, Shape *o, bool protect = true)
{
    if (!c || !s) return ABFT_EINVAL;
    if (dt != ABFT_I8 && dt != ABFT_BF16 && dt != ABFT_F16) return ABFT_EINVAL;
    if (s->M < 1 || s->N < 1 || s->K < 1 || s->batch < 1) return ABFT_ESHAPE;
    if (s->M > (1 << 30) || s->N > (1 << 30) || s->K > (1 << 30) || s->batch > 65535) return ABFT_ESHAPE;
    if (s->transB != 0 && s->transB != 1) return ABFT_EINVAL;
    const int es = elem_size(dt), os = out_size(dt);
    if (dt == ABFT_I8 && s->K >= (1 << 17)) return ABFT_ESHAPE;       // K * 2^14 must stay below 2^31
    if (protect && (need & 1) && s->K > protect_max_k(dt)) return ABFT_ESHAPE;   // deeper than the protected GEMM covers
    if ((need & 1) && s->lda < s->K) return ABFT_ESHAPE;
    if ((need & 2) && s->ldb < (s->transB ? s->K : s->N)) return ABFT_ESHAPE;
    if ((need & 4) && s->ldc < s->N) return ABFT_ESHAPE;
    if ((need & 1) && (s->lda * es) % 16) return ABFT_EALIGN;
    if ((need & 2) && (s->ldb * es) % 16) return ABFT_EALIGN;
    if ((need & 4) && (s->ldc * os) % 16) return ABFT_EALIGN;
    if (s->batch > 1) {
        if ((need & 1) && (s->strideA < 0 || (s->strideA * es) % 16)) return ABFT_EALIGN;
        if ((need & 2) && (s->strideB < 0 || (s->strideB * es) % 16)) return ABFT_EALIGN;
        if ((need & 4) && (s->strideC < s->M * s->ldc || (s->strideC * os) % 16)) return ABFT_EALIGN;
    }
    const int64_t Kp = round_up(s->K, SLAB_BYTES / es);
    if (s->batch * s->M > c->cfg.max_rows || s->batch * s->N > c->cfg.max_cols ||
        s->batch * Kp > c->cfg.max_depth || s->batch > c->cfg.max_batch)
        return ABFT_EWORKSPACE;
    o->M = (int)s->M; o->N = (int)s->N; o->K = (int)s->K; o->batch = (int)s->batch; o->transB = s->transB;
    o->lda = s->lda; o->ldb = s->ldb; o->ldc = s->ldc;
    o->sA = s->batch > 1 ? s->strideA : 0;
    o->sB = s->batch > 1 ? s->strideB : 0;
    o->sC = s->batch > 1 ? s->strideC : 0;
    o->Kp = (int)Kp;
    return ABFT_OK;
}

static void carve(const abft_ctx *c, int dt, const Shape &s, Workspace *w)
{
    const size_t bK = (size_t)s.batch * s.K, bM = (size_t)s.batch * s.M, bN = (size_t)s.batch * s.N;
    const size_t D = (size_t)c->cfg.max_depth, Bt = (size_t)c->cfg.max_batch;
    w->b_sum = c->pool_depth + (size_t)c->bslot * c->bslot_words;
    w->b_max = w->b_sum + D;
    uint32_t *pb = c->pool_batch;
    w->maxabs = (float *)pb;                  pb += 2 * Bt;
    w->tau = (float *)pb;                     pb += Bt;
    w->s_pred = pb;
    w->cc_pred = c->pool_cols;
    // the region the protected GEMM accumulates into (must be zero before it)
    w->cc_obs = c->pool_obs + (size_t)c->cur * c->region_words;
    w->rc_obs = w->cc_obs + bN;
    w->rc_pred = w->rc_obs + bM;
    w->a_sum = w->rc_pred + bM;
    w->a_max = w->a_sum + bK;
    w->cc_sto = w->a_max + s.batch;
    w->rc_sto = w->cc_sto + bN;
    w->c_max = w->rc_sto + bM;
    w->zero_words = 2 * bN + 3 * bM + bK + 2 * (size_t)s.batch;
    w->cc_vobs = c->pool_vobs + (size_t)c->vcur * c->vregion_words;
    w->rc_vobs = w->cc_vobs + bN;
    w->fix_tiles = c->fix_tiles;
    w->fix_count = c->small;
    w->cmp_ticket = c->small + 4;
    w->bias = nullptr;
    w->a_given = w->amax_given = nullptr;
    (void)dt;
}

static bool same_b(const abft_shape &x, const abft_shape &y)
{
    return x.N == y.N && x.K == y.K && x.batch == y.batch && x.transB == y.transB && x.ldb == y.ldb &&
           (x.batch == 1 || x.strideB == y.strideB);
}
static bool same_out(const abft_shape &x, const abft_shape &y)
{
    return x.M == y.M && x.N == y.N && x.batch == y.batch;
}
// abft_correct recomputes tiles from A and B: the operand geometry must be the one the predictions
// were formed with
static bool same_problem(const abft_shape &x, const abft_shape &y)
{
    return same_out(x, y) && x.K == y.K && x.transB == y.transB && x.lda == y.lda && x.ldb == y.ldb &&
           x.ldc == y.ldc &&
           (x.batch == 1 || (x.strideA == y.strideA && x.strideB == y.strideB && x.strideC == y.strideC));
}
static bool same_c_layout(const abft_shape &x, const abft_shape &y)
{
    return same_out(x, y) && x.ldc == y.ldc && (x.batch == 1 || x.strideC == y.strideC);
}

static int check_verdict(const abft_result *r, Verdict *v)
{
    if (!r || !r->row_flag || !r->col_flag || !r->counts) return ABFT_EINVAL;
    if (!(r->tau >= 0.f) || !(r->tau_cols >= 0.f)) return ABFT_EINVAL;
    v->row_flag = r->row_flag; v->col_flag = r->col_flag; v->counts = r->counts; v->tau_override = r->tau;
    v->tau_override_cols = r->tau_cols;
    return ABFT_OK;
}

#define HIP_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return fail_hip(ctx, e_); } while (0)

// A re-sum of stored C accumulates into the re-summing region the previous one did not use; the
// compare that follows clears that previous region.  Returns what the caller passes on.
struct ResumPlan { size_t stale; uint32_t *other; size_t other_words; };
// While a stream is being captured into a graph, what the host knows about the regions describes
// the moment of capture, not the moment of a replay (a replayed call finds the region it
// accumulates into as its own previous replay left it).  Calls enqueued under capture therefore
// clear everything they accumulate into themselves; the alternation between two regions, which
// saves that clearing, is for calls that run once.
static bool capturing(hipStream_t st)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(st, &cs) == hipSuccess && cs == hipStreamCaptureStatusActive;
}
// Once a call of a context has been captured, replays run at times the host does not see, so
// what the host knows about "which region is clean" is worth nothing any more, for captured and
// for eager calls alike.  From then on (sticky) the context stops alternating: every call works
// on the regions in use at that moment, clears what it accumulates into itself before it starts
// and clears nothing else.  The context then behaves like one with a single set of regions: the
// last call that ran, eager or replayed, is the one whose vectors it holds.
static bool in_graph_mode(abft_ctx *ctx, hipStream_t st)
{
    if (!ctx->graph_mode && capturing(st)) ctx->graph_mode = true;
    return ctx->graph_mode;
}

static ResumPlan begin_resum(abft_ctx *ctx, size_t words, hipStream_t st)
{
    if (in_graph_mode(ctx, st)) {
        ResumPlan p;
        p.stale = words > ctx->vdirty[ctx->vcur] ? words : ctx->vdirty[ctx->vcur];
        if (p.stale > ctx->vregion_words) p.stale = ctx->vregion_words;
        p.other = nullptr;
        p.other_words = 0;
        ctx->vdirty[ctx->vcur] = ctx->vregion_words;
        return p;
    }
    const int prev = ctx->vcur;
    ctx->vcur ^= 1;
    ResumPlan p;
    p.stale = ctx->vdirty[ctx->vcur];
    p.other = ctx->pool_vobs + (size_t)prev * ctx->vregion_words;
    p.other_words = ctx->vdirty[prev];
    // until the kernels are enqueued both count as dirty; end_resum settles it
    ctx->vdirty[ctx->vcur] = ctx->vregion_words;
    ctx->vdirty[prev] = ctx->vregion_words;
    (void)words;
    return p;
}
static void end_resum(abft_ctx *ctx, size_t words)
{
    ctx->vdirty[ctx->vcur] = words;
    if (!ctx->graph_mode) ctx->vdirty[ctx->vcur ^ 1] = 0;
}

// A pass over B accumulates into the slot that is not in use; that slot is clean unless two
// passes follow each other without a protected GEMM in between (whose finish kernel cleans it).
static int begin_b_pass(abft_ctx *ctx, hipStream_t st)
{
    const bool gm = in_graph_mode(ctx, st);
    const int target = gm ? ctx->bslot : ctx->bslot ^ 1;
    if (!ctx->bclean[target] || gm)
        HIP_TRY(launch_zero(ctx->pool_depth + (size_t)target * ctx->bslot_words, ctx->bslot_words, st));
    ctx->bclean[target] = false;
    ctx->bslot = target;
    return ABFT_OK;
}

extern "C" int abft_encode_b(abft_ctx *ctx, const void *B, abft_dtype dtype, const abft_shape *s, void *stream)
{
    Shape sh;
    int rc = check_shape(ctx, dtype, s, 2, &sh);
    if (rc) return rc;
    if (!B) return ABFT_EINVAL;
    if (!aligned16(B)) return ABFT_EALIGN;
    ctx->b_valid = false;
    rc = begin_b_pass(ctx, (hipStream_t)stream);
    if (rc) return rc;
    Workspace w;
    carve(ctx, dtype, sh, &w);
    HIP_TRY(launch_encode_b(dtype, B, sh, w, nullptr, 0, (hipStream_t)stream));
    ctx->b_valid = true;
    ctx->b_dt = dtype;
    ctx->b_shape = *s;
    return ABFT_OK;
}

// The kernels of a protected GEMM, tiled path: pass over B (unless its encoding is cached), GEMM,
// finish.  The call accumulates into the region the previous protected call did not use.  It is
// clean unless a call failed half way; the region of the previous call is cleared by this
// call's finish kernel.  So a call with a cached B checksum is two kernels: GEMM, finish.
static int enqueue_tiled(abft_ctx *ctx, int dtype, bool cached, bool stored, const void *A, const void *B, void *C,
                         const Shape &sh, Workspace *w, const Verdict &v, const InjectArm &arm, hipEvent_t *ev,
                         hipStream_t st)
{
    const bool gm = in_graph_mode(ctx, st);
    const int prev = ctx->cur;
    if (!gm) ctx->cur ^= 1;
    if (!cached) {
        int rc = begin_b_pass(ctx, st);
        if (rc) return rc;
    }
    const uint32_t *bias = w->bias, *a_given = w->a_given, *amax_given = w->amax_given;
    carve(ctx, dtype, sh, w);
    w->bias = bias; w->a_given = a_given; w->amax_given = amax_given;
    uint32_t *prev_base = ctx->pool_obs + (size_t)prev * ctx->region_words;
    size_t stale = ctx->dirty[ctx->cur];
    if (gm && stale < w->zero_words) stale = w->zero_words;
    ctx->dirty[ctx->cur] = ctx->region_words;            // until everything below is enqueued
    if (!cached) HIP_TRY(launch_encode_b(dtype, B, sh, *w, w->cc_obs, stale, st));
    else if (stale) HIP_TRY(launch_zero(w->cc_obs, stale, st));
    if (ev) HIP_TRY(hipEventRecord(ev[1], st));
    ctx->sto_valid = false;
    HIP_TRY(launch_gemm(dtype, true, stored, A, B, C, sh, *w, arm, st));
    if (ctx->done_event && !gm) HIP_TRY(hipEventRecord(ctx->done_event, st));
    if (ev) HIP_TRY(hipEventRecord(ev[2], st));
    if (gm) {
        HIP_TRY(launch_finish(dtype, B, sh, *w, v, nullptr, 0, nullptr, 0, st));
        ctx->dirty[ctx->cur] = w->zero_words;
    } else {
        const size_t prev_dirty = ctx->dirty[prev];
        ctx->dirty[prev] = ctx->region_words;
        // the finish kernel also cleans the b slot that is not in use (for the next pass over B)
        const int other = ctx->bslot ^ 1;
        uint32_t *other_base = ctx->pool_depth + (size_t)other * ctx->bslot_words;
        HIP_TRY(launch_finish(dtype, B, sh, *w, v, prev_base, prev_dirty, ctx->bclean[other] ? nullptr : other_base,
                              ctx->bslot_words, st));
        ctx->bclean[other] = true;
        ctx->dirty[prev] = 0;
        ctx->dirty[ctx->cur] = w->zero_words;
    }
    if (ev) HIP_TRY(hipEventRecord(ev[3], st));
    return ABFT_OK;
}

// A batch of small problems: one kernel does everything and writes the workspace vectors with
// plain stores, into the region and the b slot in use (nothing has to start at zero; what it
// leaves there counts as dirty for the tiled path).
static int enqueue_item(abft_ctx *ctx, int dtype, bool cached, bool stored, const void *A, const void *B, void *C,
                        const Shape &sh, const Workspace &w, const Verdict &v, const InjectArm &arm, hipEvent_t *ev,
                        hipStream_t st)
{
    if (ev) HIP_TRY(hipEventRecord(ev[1], st));
    if (!cached) ctx->bclean[ctx->bslot] = false;
    if (ctx->dirty[ctx->cur] < w.zero_words) ctx->dirty[ctx->cur] = w.zero_words;
    ctx->sto_valid = false;
    HIP_TRY(launch_gemm_item(dtype, true, cached, stored, A, B, C, sh, w, &v, arm, st));
    if (ctx->done_event && !in_graph_mode(ctx, st)) HIP_TRY(hipEventRecord(ctx->done_event, st));
    if (ev) { HIP_TRY(hipEventRecord(ev[2], st)); HIP_TRY(hipEventRecord(ev[3], st)); }
    return ABFT_OK;
}

// The context now holds the row / column sums of this stored C.
static void note_vobs(abft_ctx *ctx, const void *C, const abft_shape *s, hipStream_t st)
{
    ctx->vobs_valid = true;
    ctx->vobs_captured = capturing(st);
    ctx->vobs_C = C;
    ctx->vobs_ldc = s->ldc;
    ctx->vobs_strideC = s->batch > 1 ? s->strideC : 0;
}
// May a correction bring those sums up to date in place instead of summing the whole C again?
// Only if they belong to this C, and, once a graph is in play, only inside the captured sequence
// that formed them (what an eager call finds in the region may be a replay's).
static bool vobs_usable(const abft_ctx *ctx, const void *C, const abft_shape *s, hipStream_t st)
{
    if (!ctx->vobs_valid || ctx->vobs_C != C || ctx->vobs_ldc != s->ldc ||
        ctx->vobs_strideC != (s->batch > 1 ? s->strideC : 0))
        return false;
    if (!ctx->graph_mode) return true;
    return ctx->vobs_captured && capturing(st);
}

static int gemm_impl(abft_ctx *ctx, const void *A, const void *B, const void *bias, void *C, abft_dtype dtype, int mode,
                     const abft_shape *s, const abft_result *r, void *stream);

extern "C" int abft_gemm(abft_ctx *ctx, const void *A, const void *B, void *C, abft_dtype dtype, int mode,
                         const abft_shape *s, const abft_result *r, void *stream)
{
    return gemm_impl(ctx, A, B, nullptr, C, dtype, mode, s, r, stream);
}

extern "C" int abft_gemm_bias(abft_ctx *ctx, const void *A, const void *B, const void *bias, void *C,
                              abft_dtype dtype, int mode, const abft_shape *s, const abft_result *r, void *stream)
{
    if (!bias) return ABFT_EINVAL;
    if (((uintptr_t)bias & 3u) != 0) return ABFT_EALIGN;
    return gemm_impl(ctx, A, B, bias, C, dtype, mode, s, r, stream);
}

static int gemm_impl(abft_ctx *ctx, const void *A, const void *B, const void *bias, void *C, abft_dtype dtype, int mode,
                     const abft_shape *s, const abft_result *r, void *stream)
{
    const int base = mode & ABFT_MODE_MASK;
    if (base != ABFT_OFF && base != ABFT_DETECT && base != ABFT_DETECT_CORRECT) return ABFT_EINVAL;
    if (mode & ~(ABFT_MODE_MASK | ABFT_B_CHECKSUM_CACHED | ABFT_STORED_SUMS | ABFT_A_CHECKSUM_GIVEN)) return ABFT_EINVAL;
    Shape sh;
    int rc = check_shape(ctx, dtype, s, 7, &sh, base != ABFT_OFF);
    if (rc) return rc;
    if (!A || !B || !C) return ABFT_EINVAL;
    if (!aligned16(A) || !aligned16(B) || !aligned16(C)) return ABFT_EALIGN;
    hipStream_t st = (hipStream_t)stream;
    Workspace w;
    carve(ctx, dtype, sh, &w);
    w.bias = (const uint32_t *)bias;
    const bool given = base != ABFT_OFF && (mode & ABFT_A_CHECKSUM_GIVEN) != 0;
    if (given) {
        if (!ctx->given_a) return ABFT_ESTATE;                       // abft_supply_a first
        // without max|A| there is no default tolerance: the caller must bring one
        if (dtype != ABFT_I8 && !ctx->given_amax && !(r && r->tau > 0.f)) return ABFT_EINVAL;
        w.a_given = (const uint32_t *)ctx->given_a;
        w.amax_given = (const uint32_t *)ctx->given_amax;
    }
    InjectArm arm = ctx->arm;
    if (arm.batch >= 0 && (arm.batch >= sh.batch || arm.row >= sh.M || arm.col >= sh.N)) return ABFT_EINVAL;

    if (base == ABFT_OFF) {
        ctx->arm.batch = -1;
        hipEvent_t *ev = (ctx->prof_ev && ctx->prof_n < ctx->prof_cap) ? ctx->prof_ev + 4 * ctx->prof_n : nullptr;
        if (ev) { HIP_TRY(hipEventRecord(ev[0], st)); HIP_TRY(hipEventRecord(ev[1], st)); }
        HIP_TRY(launch_gemm(dtype, false, false, A, B, C, sh, w, arm, st));
        if (ctx->done_event && !capturing(st)) HIP_TRY(hipEventRecord(ctx->done_event, st));
        if (ev) { HIP_TRY(hipEventRecord(ev[2], st)); HIP_TRY(hipEventRecord(ev[3], st)); ctx->prof_n++; }
        return ABFT_OK;
    }
    Verdict v;
    rc = check_verdict(r, &v);
    if (rc) return rc;
    const bool cached = (mode & ABFT_B_CHECKSUM_CACHED) != 0;
    if (cached && !(ctx->b_valid && ctx->b_dt == (int)dtype && same_b(ctx->b_shape, *s))) return ABFT_ESTATE;
    ctx->pred_valid = false;
    ctx->vobs_valid = false;
    if (!cached) ctx->b_valid = false;
    ctx->arm.batch = -1;
    hipEvent_t *ev = (ctx->prof_ev && ctx->prof_n < ctx->prof_cap) ? ctx->prof_ev + 4 * ctx->prof_n : nullptr;
    if (ev) HIP_TRY(hipEventRecord(ev[0], st));
    const bool stored = (mode & ABFT_STORED_SUMS) != 0;
    const bool item = !bias && !given && gemm_item_eligible(dtype, sh, stored);
    rc = item ? enqueue_item(ctx, dtype, cached, stored, A, B, C, sh, w, v, arm, ev, st)
              : enqueue_tiled(ctx, dtype, cached, stored, A, B, C, sh, &w, v, arm, ev, st);
    if (rc) return rc;
    if (ev) ctx->prof_n++;
    ctx->b_valid = true;
    ctx->b_dt = dtype;
    ctx->b_shape = *s;
    ctx->pred_valid = true;
    ctx->pred_dt = dtype;
    ctx->pred_shape = *s;
    ctx->pred_bias = bias;
    if (given) ctx->given_a = ctx->given_amax = nullptr;              // consumed
    // a correction inside this call replaces values the stored-side sums already contain
    ctx->sto_valid = stored && base == ABFT_DETECT;
    if (base == ABFT_DETECT_CORRECT) {
        const size_t words = (size_t)sh.batch * ((size_t)sh.M + sh.N);
        const ResumPlan rp = begin_resum(ctx, words, st);
        carve(ctx, dtype, sh, &w);
        w.bias = (const uint32_t *)bias;
        const bool clear_list = ctx->list_dirty || ctx->graph_mode;
        ctx->list_dirty = true;
        // a clean call (the common case) must not pay for a pass over the whole stored C: the
        // re-sum and the compare behind the recompute do nothing when no tile was listed
        HIP_TRY(launch_correct(dtype, A, B, C, sh, w, v, false, clear_list, false, rp.stale, rp.other, rp.other_words, st,
                               true));
        ctx->list_dirty = false;
        end_resum(ctx, words);
        ctx->vobs_valid = false;                 // whether the sums were formed is known on the device only
    }
    return ABFT_OK;
}

// ------------------------------------------------------------------------------------------
// abft_gemm for callers that cannot allocate device memory (code under graph capture, serving
// loops, harnesses that forbid it): the workspace is a fixed array in the library's device image
// instead of the pools abft_create allocates.  Every GPU holds its own copy of the array, at its
// own address, from the moment the library is loaded until the process ends.
constexpr int64_t STATIC_MAX_ROWS = ABFT_STATIC_MAX_ROWS, STATIC_MAX_COLS = ABFT_STATIC_MAX_COLS,
                  STATIC_MAX_DEPTH = ABFT_STATIC_MAX_DEPTH, STATIC_MAX_BATCH = ABFT_STATIC_MAX_BATCH;
constexpr int64_t STATIC_DEPTH_WORDS = STATIC_MAX_DEPTH + (int64_t)SLAB_BYTES * STATIC_MAX_BATCH;   // as abft_create rounds it
// every pool starts on a 256-byte boundary
constexpr size_t STATIC_SCRATCH_WORDS =
    pool_total_words(STATIC_MAX_ROWS, STATIC_MAX_COLS, STATIC_DEPTH_WORDS, STATIC_MAX_BATCH) + N_POOLS * 64;
static __device__ __align__(256) uint32_t scratch[STATIC_SCRATCH_WORDS];

constexpr int STATIC_MAX_DEVICES = 32;
static abft_ctx g_static_ctx[STATIC_MAX_DEVICES];     // static storage: zero-initialised
static bool g_static_ready[STATIC_MAX_DEVICES];
static std::mutex g_static_lock;

extern "C" int abft_gemm_static(const void *A, const void *B, void *C, abft_dtype dtype, int mode,
                                const abft_shape *s, const abft_result *r, void *stream)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return ABFT_EHIP;
    abft_ctx *ctx = &g_static_ctx[dev];
    {
        std::lock_guard<std::mutex> hold(g_static_lock);
        if (!g_static_ready[dev]) {
            // `scratch` in host code is a stand-in for the symbol, not a device address: ask the
            // runtime where this device's copy of the array lives, once, and use that pointer.
            uint32_t *base = nullptr;
            hipError_t e = hipGetSymbolAddress((void **)&base, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !base) { ctx->last_hip = (int)e; return ABFT_EHIP; }
            memset(ctx, 0, sizeof(*ctx));
            ctx->is_static = true;
            ctx->cfg.max_rows = STATIC_MAX_ROWS;
            ctx->cfg.max_cols = STATIC_MAX_COLS;
            ctx->cfg.max_depth = STATIC_DEPTH_WORDS;
            ctx->cfg.max_batch = STATIC_MAX_BATCH;
            ctx->cfg.device = dev;
            ctx->arm.batch = -1;
            size_t words[N_POOLS];
            pool_words(STATIC_MAX_ROWS, STATIC_MAX_COLS, STATIC_DEPTH_WORDS, STATIC_MAX_BATCH, words);
            void **slot[N_POOLS];
            pool_slots(ctx, slot);
            size_t off = 0;
            for (int i = 0; i < N_POOLS; ++i) {
                *slot[i] = base + off;
                off += (words[i] + 63) / 64 * 64;
            }
            if (off > STATIC_SCRATCH_WORDS) return ABFT_EWORKSPACE;
            // The array is zero when the library is loaded; whatever an earlier user of this process
            // left in it is cleared here, by a kernel on the caller's stream (no memset node: the
            // call may be under capture).
            e = launch_zero(base, STATIC_SCRATCH_WORDS, (hipStream_t)stream);
            if (e != hipSuccess) { ctx->last_hip = (int)e; return ABFT_EHIP; }
            start_clean(ctx);
            g_static_ready[dev] = true;
        }
    }
    return abft_gemm(ctx, A, B, C, dtype, mode, s, r, stream);
}

extern "C" int abft_gemm_done_event(abft_ctx *ctx, void *event)
{
    if (!ctx) return ABFT_EINVAL;
    ctx->done_event = (hipEvent_t)event;
    return ABFT_OK;
}

extern "C" int abft_supply_a(abft_ctx *ctx, const void *a, const void *amax)
{
    if (!ctx || !a) return ABFT_EINVAL;
    if (((uintptr_t)a & 3u) || ((uintptr_t)amax & 3u)) return ABFT_EALIGN;
    ctx->given_a = a;
    ctx->given_amax = amax;
    return ABFT_OK;
}

extern "C" int abft_verify(abft_ctx *ctx, const void *C, abft_dtype dtype, const abft_shape *s,
                           const abft_result *r, void *stream)
{
    Shape sh;
    int rc = check_shape(ctx, dtype, s, 4, &sh);
    if (rc) return rc;
    if (!C) return ABFT_EINVAL;
    if (!aligned16(C)) return ABFT_EALIGN;
    Verdict v;
    rc = check_verdict(r, &v);
    if (rc) return rc;
    if (!(ctx->pred_valid && ctx->pred_dt == (int)dtype && same_c_layout(ctx->pred_shape, *s))) return ABFT_ESTATE;
    hipStream_t st = (hipStream_t)stream;
    const size_t words = (size_t)sh.batch * ((size_t)sh.M + sh.N);
    ctx->vobs_valid = false;
    const ResumPlan rp = begin_resum(ctx, words, st);
    Workspace w;
    carve(ctx, dtype, sh, &w);
    if (rp.stale) HIP_TRY(launch_zero(w.cc_vobs, rp.stale, st));
    HIP_TRY(launch_verify_sums(dtype, C, sh, w, st));
    HIP_TRY(launch_compare(dtype, sh, w, v, false, ctx->sto_valid, rp.other, rp.other_words, st));
    end_resum(ctx, words);
    note_vobs(ctx, C, s, st);
    return ABFT_OK;
}

extern "C" int abft_correct(abft_ctx *ctx, const void *A, const void *B, void *C, abft_dtype dtype,
                            const abft_shape *s, const abft_result *r, void *stream)
{
    Shape sh;
    int rc = check_shape(ctx, dtype, s, 7, &sh);
    if (rc) return rc;
    if (!A || !B || !C) return ABFT_EINVAL;
    if (!aligned16(A) || !aligned16(B) || !aligned16(C)) return ABFT_EALIGN;
    Verdict v;
    rc = check_verdict(r, &v);
    if (rc) return rc;
    if (!(ctx->pred_valid && ctx->pred_dt == (int)dtype && same_problem(ctx->pred_shape, *s))) return ABFT_ESTATE;
    hipStream_t st = (hipStream_t)stream;
    const bool clear_list = ctx->list_dirty || in_graph_mode(ctx, st);
    Workspace w;
    if (vobs_usable(ctx, C, s, st)) {
        // abft_verify (or an earlier correction) left the sums of this stored C: they are brought up
        // to date in place, for the rows and columns of the recomputed tiles only
        carve(ctx, dtype, sh, &w);
        w.bias = (const uint32_t *)ctx->pred_bias;
        ctx->list_dirty = true;
        ctx->vobs_valid = false;
        HIP_TRY(launch_correct(dtype, A, B, C, sh, w, v, ctx->sto_valid, clear_list, true, 0, nullptr, 0, st));
        ctx->list_dirty = false;
        ctx->vobs_valid = true;
        return ABFT_OK;
    }
    ctx->vobs_valid = false;
    const size_t words = (size_t)sh.batch * ((size_t)sh.M + sh.N);
    const ResumPlan rp = begin_resum(ctx, words, st);
    carve(ctx, dtype, sh, &w);
    w.bias = (const uint32_t *)ctx->pred_bias;
    ctx->list_dirty = true;
    HIP_TRY(launch_correct(dtype, A, B, C, sh, w, v, ctx->sto_valid, clear_list, false, rp.stale, rp.other,
                           rp.other_words, st));
    ctx->list_dirty = false;
    end_resum(ctx, words);
    note_vobs(ctx, C, s, st);
    return ABFT_OK;
}

extern "C" int abft_correct_checksum(abft_ctx *ctx, void *C, abft_dtype dtype, const abft_shape *s,
                                     const abft_result *r, void *stream)
{
    Shape sh;
    int rc = check_shape(ctx, dtype, s, 4, &sh);
    if (rc) return rc;
    if (dtype != ABFT_I8) return ABFT_EINVAL;     // a rounded sum cannot restore the stored bits
    if (!C) return ABFT_EINVAL;
    if (!aligned16(C)) return ABFT_EALIGN;
    Verdict v;
    rc = check_verdict(r, &v);
    if (rc) return rc;
    if (!(ctx->pred_valid && ctx->pred_dt == (int)dtype && same_out(ctx->pred_shape, *s))) return ABFT_ESTATE;
    if (!vobs_usable(ctx, C, s, (hipStream_t)stream)) return ABFT_ESTATE;     // needs the re-summed stored C of abft_verify
    Workspace w;
    carve(ctx, dtype, sh, &w);
    HIP_TRY(launch_arith_fix(C, sh, w, v, (hipStream_t)stream));
    return ABFT_OK;
}

extern "C" int abft_discrepancy(abft_ctx *ctx, abft_dtype dtype, const abft_shape *s, int source, float *stats,
                                void *stream)
{
    Shape sh;
    int rc = check_shape(ctx, dtype, s, 0, &sh);
    if (rc) return rc;
    if (dtype == ABFT_I8) return ABFT_EINVAL;              // integers compare for equality: nothing to fit
    if (!stats || (source != ABFT_DISC_FUSED && source != ABFT_DISC_STORED)) return ABFT_EINVAL;
    if (!(ctx->pred_valid && ctx->pred_dt == (int)dtype && same_out(ctx->pred_shape, *s))) return ABFT_ESTATE;
    if (source == ABFT_DISC_STORED && !ctx->vobs_valid) return ABFT_ESTATE;
    Workspace w;
    carve(ctx, dtype, sh, &w);
    HIP_TRY(launch_discrepancy(sh, w, source == ABFT_DISC_STORED, stats, (hipStream_t)stream));
    return ABFT_OK;
}

extern "C" int abft_inject(abft_ctx *ctx, void *C, abft_dtype dtype, const abft_shape *s, int64_t batch_idx,
                           int64_t row, int64_t col, int bit, int where, void *stream)
{
    Shape sh;
    if (where == ABFT_INJECT_OPERAND_A || where == ABFT_INJECT_OPERAND_B) {
        // a bit of an element of the stored operand array: A is M x K; B is N x K or K x N as stored
        const bool isA = where == ABFT_INJECT_OPERAND_A;
        int rc = check_shape(ctx, dtype, s, isA ? 1 : 2, &sh, false);
        if (rc) return rc;
        if (!C) return ABFT_EINVAL;
        const int64_t rows = isA ? sh.M : (sh.transB ? sh.N : sh.K), cols = isA ? sh.K : (sh.transB ? sh.K : sh.N);
        if (batch_idx < 0 || batch_idx >= sh.batch || row < 0 || row >= rows || col < 0 || col >= cols) return ABFT_EINVAL;
        if (bit < 0 || bit >= 8 * elem_size(dtype)) return ABFT_EINVAL;
        const long idx = batch_idx * (isA ? sh.sA : sh.sB) + row * (isA ? sh.lda : sh.ldb) + col;
        HIP_TRY(launch_flip_at(C, idx, elem_size(dtype), bit, (hipStream_t)stream));
        return ABFT_OK;
    }
    int rc = check_shape(ctx, dtype, s, where == ABFT_INJECT_STORED_C ? 4 : 0, &sh);
    if (rc) return rc;
    if (batch_idx < 0 || batch_idx >= sh.batch || row < 0 || row >= sh.M || col < 0 || col >= sh.N)
        return ABFT_EINVAL;
    if (where == ABFT_INJECT_ACCUMULATOR) {
        if (bit < 0 || bit > 31) return ABFT_EINVAL;
        ctx->arm.batch = (int)batch_idx; ctx->arm.row = (int)row; ctx->arm.col = (int)col; ctx->arm.bit = bit;
        return ABFT_OK;
    }
    if (where != ABFT_INJECT_STORED_C) return ABFT_EINVAL;
    if (!C) return ABFT_EINVAL;
    if (bit < 0 || bit >= 8 * out_size(dtype)) return ABFT_EINVAL;
    HIP_TRY(launch_flip(C, dtype, sh, batch_idx, row, col, bit, (hipStream_t)stream));
    if (C == ctx->vobs_C) ctx->vobs_valid = false;     // the sums the context holds describe C before the flip
    return ABFT_OK;
}

extern "C" int abft_workspace(abft_ctx *ctx, int which, const abft_shape *s, void **ptr, int64_t *count)
{
    if (!ptr || !count || !s) return ABFT_EINVAL;
    Shape sh;
    // dtype does not change the carving except through Kp; take the widest (1-byte elements)
    int rc = check_shape(ctx, ABFT_I8, s, 0, &sh);
    if (rc == ABFT_ESHAPE && s->K >= (1 << 17)) rc = check_shape(ctx, ABFT_BF16, s, 0, &sh);
    if (rc) return rc;
    Workspace w;
    carve(ctx, 0, sh, &w);
    const int64_t b = sh.batch;
    switch (which) {
    case ABFT_WS_A_SUM:   *ptr = w.a_sum;   *count = b * sh.K; break;
    case ABFT_WS_B_SUM:   *ptr = w.b_sum;   *count = b * sh.K; break;
    case ABFT_WS_CC_PRED: *ptr = w.cc_pred; *count = b * sh.N; break;
    case ABFT_WS_RC_PRED: *ptr = w.rc_pred; *count = b * sh.M; break;
    case ABFT_WS_CC_OBS:  *ptr = w.cc_obs;  *count = b * sh.N; break;
    case ABFT_WS_RC_OBS:  *ptr = w.rc_obs;  *count = b * sh.M; break;
    case ABFT_WS_CC_VOBS: *ptr = w.cc_vobs; *count = b * sh.N; break;
    case ABFT_WS_RC_VOBS: *ptr = w.rc_vobs; *count = b * sh.M; break;
    case ABFT_WS_TAU:     *ptr = w.tau;     *count = b; break;
    case ABFT_WS_S_PRED:  *ptr = w.s_pred;  *count = b; break;
    case ABFT_WS_MAXABS:  *ptr = w.maxabs;  *count = 2 * b; break;
    case ABFT_WS_CC_STO:  *ptr = w.cc_sto;  *count = b * sh.N; break;
    case ABFT_WS_RC_STO:  *ptr = w.rc_sto;  *count = b * sh.M; break;
    case ABFT_WS_C_MAX:   *ptr = w.c_max;   *count = b; break;
    default: return ABFT_EINVAL;
    }
    return ABFT_OK;
}

static void prof_free(abft_ctx *c)
{
    if (c->prof_ev) {
        for (int i = 0; i < 4 * c->prof_cap; ++i)
            if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
        delete[] c->prof_ev;
    }
    c->prof_ev = nullptr;
    c->prof_cap = c->prof_n = 0;
}

extern "C" int abft_profile_begin(abft_ctx *ctx, int max_calls)
{
    if (!ctx || max_calls < 1 || max_calls > 100000) return ABFT_EINVAL;
    prof_free(ctx);
    ctx->prof_ev = new (std::nothrow) hipEvent_t[4 * (size_t)max_calls];
    if (!ctx->prof_ev) return ABFT_EINVAL;
    memset(ctx->prof_ev, 0, sizeof(hipEvent_t) * 4 * (size_t)max_calls);
    ctx->prof_cap = max_calls;
    for (int i = 0; i < 4 * max_calls; ++i) {
        hipError_t e = hipEventCreate(&ctx->prof_ev[i]);
        if (e != hipSuccess) { prof_free(ctx); return fail_hip(ctx, e); }
    }
    return ABFT_OK;
}

extern "C" int abft_profile_end(abft_ctx *ctx, double ms[4], int *calls)
{
    if (!ctx || !ms || !calls) return ABFT_EINVAL;
    if (!ctx->prof_ev) return ABFT_ESTATE;
    double sum[4] = {0, 0, 0, 0};
    const int n = ctx->prof_n;
    for (int i = 0; i < n; ++i) {
        hipEvent_t *ev = ctx->prof_ev + 4 * i;
        hipError_t e = hipEventSynchronize(ev[3]);
        if (e != hipSuccess) { prof_free(ctx); return fail_hip(ctx, e); }
        float t;
        for (int q = 0; q < 3; ++q) {
            e = hipEventElapsedTime(&t, ev[q], ev[q + 1]);
            if (e != hipSuccess) { prof_free(ctx); return fail_hip(ctx, e); }
            sum[q] += t;
        }
        e = hipEventElapsedTime(&t, ev[0], ev[3]);
        if (e != hipSuccess) { prof_free(ctx); return fail_hip(ctx, e); }
        sum[3] += t;
    }
    for (int q = 0; q < 4; ++q) ms[q] = n ? sum[q] / n : 0.0;
    *calls = n;
    prof_free(ctx);
    return ABFT_OK;
}

extern "C" int abft_mfma_peak(abft_dtype dtype, double seconds, double *tera_ops, double *clock_mhz)
{
    if (!tera_ops || !clock_mhz || !(seconds > 0.0) || seconds > 2.0) return ABFT_EINVAL;
    if (dtype != ABFT_I8 && dtype != ABFT_BF16 && dtype != ABFT_F16) return ABFT_EINVAL;
    hipError_t e = hipSuccess;
    const int cus = device_cu_count(&e);
    if (e != hipSuccess || cus <= 0) return ABFT_EHIP;
    unsigned long long *clk = nullptr;
    uint32_t *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = ABFT_EHIP;
    std::vector<unsigned long long> h((size_t)2 * cus);
    const double ops_per_iter = (double)cus * 4 * 16 * 2.0 * 32 * 32 * (dtype == ABFT_I8 ? 32 : 16);
    float ms = 0.f;
    int iters = 2000;
    if (hipMalloc(&clk, sizeof(unsigned long long) * 2 * cus) != hipSuccess) goto out;
    if (hipMalloc(&sink, 256 * 4) != hipSuccess) goto out;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto out;
    // a short run sizes the long one; only the long one is reported
    for (int pass = 0; pass < 2; ++pass) {
        if (hipEventRecord(e0, nullptr) != hipSuccess) goto out;
        if (launch_mfma_peak(dtype, cus, iters, clk, sink, nullptr) != hipSuccess) goto out;
        if (hipEventRecord(e1, nullptr) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) goto out;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.f)) goto out;
        if (pass == 0) {
            double want = iters * (seconds * 1e3 / ms);
            iters = want > 5e7 ? 50000000 : (want < 2000 ? 2000 : (int)want);
        }
    }
    if (hipMemcpy(h.data(), clk, sizeof(unsigned long long) * 2 * cus, hipMemcpyDeviceToHost) != hipSuccess) goto out;
    {
        double cyc = 0, wall = 0;
        for (int i = 0; i < cus; ++i) { cyc += (double)h[2 * i]; wall += (double)h[2 * i + 1]; }
        *tera_ops = ops_per_iter * iters / (ms * 1e-3) / 1e12;
        *clock_mhz = wall > 0 ? cyc / wall * 100.0 : 0.0;      // the constant counter runs at 100 MHz
    }
    rc = ABFT_OK;
out:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (clk) (void)hipFree(clk);
    if (sink) (void)hipFree(sink);
    return rc;
}

extern "C" int abft_tile_shape(abft_dtype dtype, const abft_shape *s, int *tile_m, int *tile_n)
{
    if (!s || !tile_m || !tile_n) return ABFT_EINVAL;
    if (dtype != ABFT_I8 && dtype != ABFT_BF16 && dtype != ABFT_F16) return ABFT_EINVAL;
    Shape sh;
    memset(&sh, 0, sizeof(sh));
    sh.M = (int)s->M; sh.N = (int)s->N; sh.K = (int)s->K; sh.batch = (int)s->batch; sh.transB = s->transB;
    gemm_tile_shape(dtype, sh, tile_m, tile_n);
    return ABFT_OK;
}
