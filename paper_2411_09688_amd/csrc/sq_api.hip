// C ABI of the library: argument validation, workspace carving and kernel sequencing.  Nothing here
// computes; every step of the path runs in the kernels of the other files.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "../../include/squeezed_attention.h"
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace

int sq::set_error(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define SQ_REQUIRE_PTR(p)                                                                     \
    do {                                                                                      \
        if ((p) == nullptr) return fail(SQ_ERR_INVALID_ARG, "%s: %s is NULL", __func__, #p);  \
        if (!aligned16(p)) return fail(SQ_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", __func__, #p); \
    } while (0)
#define SQ_OPTIONAL_PTR(p)                                                                    \
    do {                                                                                      \
        if ((p) != nullptr && !aligned16(p))                                                  \
            return fail(SQ_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", __func__, #p);   \
    } while (0)
#define SQ_HIP(expr)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(SQ_ERR_HIP, "%s: %s -> %s", __func__, #expr, hipGetErrorString(e_)); \
    } while (0)

int check_shape(const sq_shape_t *sh, const char *fn, bool need_decode)
{
    if (!sh) return fail(SQ_ERR_INVALID_ARG, "%s: shape is NULL", fn);
    if (sh->B <= 0 || sh->H <= 0 || sh->L <= 0 || sh->C <= 0 || sh->Lq <= 0 || sh->U < 0)
        return fail(SQ_ERR_INVALID_ARG, "%s: non-positive dimension (B=%d H=%d L=%d C=%d Lq=%d U=%d)", fn, sh->B, sh->H,
                    sh->L, sh->C, sh->Lq, sh->U);
    if (!(sh->sm_scale == sh->sm_scale) || sh->sm_scale <= 0.0f)
        return fail(SQ_ERR_INVALID_ARG, "%s: sm_scale must be positive", fn);
    if (sh->d != sq::D) return fail(SQ_ERR_UNSUPPORTED, "%s: head dim %d not supported (d must be 128)", fn, sh->d);
    if (need_decode && sh->Lq != 1) return fail(SQ_ERR_UNSUPPORTED, "%s: decode call needs Lq == 1 (got %d)", fn, sh->Lq);
    const long long rows = (long long)sh->B * sh->H * sh->Lq;
    if (rows * (long long)sh->C > (1ll << 40) || (long long)sh->H * sh->L > (1ll << 40) || sh->L > sq::MAX_L)
        return fail(SQ_ERR_UNSUPPORTED, "%s: problem too large", fn);
    if (sh->C > sq::SELECT_MAX_C)
        return fail(SQ_ERR_UNSUPPORTED, "%s: C = %d clusters per head exceeds the supported %d", fn, sh->C,
                    sq::SELECT_MAX_C);
    return SQ_OK;
}

// The kernels are gfx950 code objects: refuse any other device with a clear message.
int check_device(const char *fn)
{
    static thread_local int ok_device = -1;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SQ_ERR_HIP, "%s: hipGetDevice -> %s", fn, hipGetErrorString(e));
    if (dev == ok_device) return SQ_OK;
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return fail(SQ_ERR_HIP, "%s: hipGetDeviceProperties -> %s", fn, hipGetErrorString(e));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(SQ_ERR_UNSUPPORTED, "%s: device %d is %s, this library is built for gfx950 only", fn, dev,
                    prop.gcnArchName);
    ok_device = dev;
    return SQ_OK;
}

size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Carves consecutive 256-byte aligned regions out of a workspace.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <typename T>
    T *take(size_t count)
    {
        T *r = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += align256(count * sizeof(T));
        return r;
    }
};

struct DecodeWs {
    sq::DecodePlan plan;
    float *partials;
};

DecodeWs carve_decode(Carver &cv, const sq_shape_t *sh, int G = 1)
{
    const size_t rows = (size_t)sh->B * sh->H * G;
    const size_t items = rows * (sq::user_chunks_for(sh->U) + sq::chunk_cap_for(sh->L));
    DecodeWs w{};
    w.plan.rec_cap = sh->C;
    w.plan.L = sh->L;
    w.plan.item_cap = (int)items;
    w.plan.rec = cv.take<int4>(rows * sh->C);
    w.plan.hdr = cv.take<int2>(rows);
    w.plan.row_items = cv.take<int2>(rows);
    w.plan.total = cv.take<int>(2);
    w.plan.item = cv.take<int2>(items * sq::ITEM_STRIDE);
    w.partials = cv.take<float>(items * sq::PART_STRIDE);
    return w;
}

// The user-key rider of a decode step's selection launch (sq_user_attn.hpp): rows = B * H * G query rows, q [rows, d],
// user keys [B * H, U, d].  Its partial results take the top rows * nuq slots of the partial buffer, which the
// work list cannot reach once it holds no user chunks (item_cap counts them).  q == nullptr without user keys.
sq::UserAttn make_user_rider(const sq_shape_t *sh, int G, const void *q, const void *K_user, const void *V_user,
                             const DecodeWs &dec)
{
    sq::UserAttn ua{};
    if (sh->U <= 0) return ua;
    const int rows = sh->B * sh->H * G, nuc = sq::user_chunks_for(sh->U);
    ua.q = static_cast<const _Float16 *>(q);
    ua.Ku = static_cast<const _Float16 *>(K_user);
    ua.Vu = static_cast<const _Float16 *>(V_user);
    ua.partials = dec.partials;
    ua.rows = rows;
    ua.U = sh->U;
    ua.G = G;
    ua.nuq = nuc;
    ua.slot_base = dec.plan.item_cap - rows * ua.nuq;
    ua.sm_scale = sh->sm_scale;
    return ua;
}

// Workspace of the whole decode step: logits, counts, plan, partials.
struct StepWs {
    float *logits;
    int32_t *n_ranges, *n_keys;
    DecodeWs dec;
};

// G: query heads per K/V head (rows = B * H * G; 1 without grouped-query attention).
StepWs carve_step(Carver &cv, const sq_shape_t *sh, int G = 1)
{
    const size_t rows = (size_t)sh->B * sh->H * G;
    StepWs w{};
    w.logits = cv.take<float>(rows * sh->C);
    w.n_ranges = cv.take<int32_t>(rows);
    w.n_keys = cv.take<int32_t>(rows);
    w.dec = carve_decode(cv, sh, G);
    return w;
}

// Workspace of the decode step through a key-index list (sq_decode_keyidx.hip): logits, counts, the rows' key-index
// lists and the partial results.
struct IndexStepWs {
    float *logits;
    int32_t *n_ranges, *n_keys;
    sq::KeyIndexPlan plan;
    float *partials;
    int user_slot_base, nuq;
};

IndexStepWs carve_step_index(Carver &cv, const sq_shape_t *sh, int G = 1)
{
    const size_t rows = (size_t)sh->B * sh->H * G;
    IndexStepWs w{};
    w.nuq = sq::user_pieces_for(sh->U);
    w.user_slot_base = sq::KI_ATTN_GRID + (int)rows;
    w.logits = cv.take<float>(rows * sh->C);
    w.n_ranges = cv.take<int32_t>(rows);
    w.n_keys = cv.take<int32_t>(rows);
    w.plan.L = sh->L;
    w.plan.row_keys = cv.take<int32_t>(rows);
    w.plan.key_idx = cv.take<int32_t>(rows * sh->L);
    w.partials = cv.take<float>(sq::keyidx_partial_slots((int)rows, w.nuq) * sq::PART_STRIDE);
    return w;
}

// The key-index step handles rows of up to KI_MAX_C clusters and calls of up to KI_MAX_ROWS query rows; anything
// larger takes the work-list kernels.
bool step_is_indexed(const sq_shape_t *sh, int G = 1)
{
    return sh->C <= sq::KI_MAX_C && (long long)sh->B * sh->H * G <= sq::KI_MAX_ROWS;
}

// Workspace of a decode step over a shared context (B >= 2): per-sequence selection outputs, then the union
// rows' plan and the partials of the shared-context kernel.
struct SharedStepWs {
    float *logits;
    int32_t *n_ranges, *n_keys;
    uint32_t *mask;
    sq::DecodePlan plan;
    float *partials;
};

// G: query rows per (sequence, head) that share the head's K/V (1, or the group size of grouped-query attention).
SharedStepWs carve_step_shared(Carver &cv, const sq_shape_t *sh, int G = 1)
{
    const size_t rows = (size_t)sh->B * sh->H * G;
    const size_t urows = (size_t)sq::seq_groups_for(sh->B * G) * sh->H;
    const size_t items = urows * ((size_t)sq::SG * sq::user_chunks_for(sh->U) + sq::chunk_cap_for(sh->L));
    SharedStepWs w{};
    w.logits = cv.take<float>(rows * sh->C);
    w.n_ranges = cv.take<int32_t>(rows);
    w.n_keys = cv.take<int32_t>(rows);
    w.mask = cv.take<uint32_t>(rows * ((sh->C + 31) / 32));
    w.plan.rec_cap = sh->C;
    w.plan.L = sh->L;
    w.plan.item_cap = (int)items;
    w.plan.rec = cv.take<int4>(urows * sh->C);
    w.plan.hdr = cv.take<int2>(urows);
    w.plan.row_items = cv.take<int2>(urows);
    w.plan.row_rank = cv.take<int>(urows);
    w.plan.total = cv.take<int>(2);
    w.plan.item = cv.take<int2>(items * sq::ITEM_STRIDE);
    w.partials = cv.take<float>(((size_t)sq::SHARED_ATTN_GRID + urows) * sq::SG * sq::PART_STRIDE);
    return w;
}

// With at least this many query rows per K/V head -- sequences over a shared context, times the query heads of a
// grouped-query group -- a decode step streams the union of their selections (shared-context kernels); with
// fewer, the overlap of the selections saves less than the union kernels cost and the per-row kernels run
// (measured at 32K context, keep 1/8: 2 sequences 65 us against 50 us per step, 6 sequences 94 against 87,
// even from 8 on; one sequence with 4 query heads per K/V head 43 us against 31 us).
constexpr int SHARED_MIN_ROWS = 8;
bool step_is_shared(const sq_shape_t *sh, int G = 1) { return sh->B * G >= SHARED_MIN_ROWS; }

// Workspace of the two-level lookup.  C1 <= C2 is not known to sq_workspace_bytes, so level-1 buffers
// are sized for C2.
struct HierWs {
    float *logits1, *logits2;   // logits2 and cand_id are in candidate order: [rows, C2] with the row's candidates first
    int32_t *cand_id;
    int32_t *nr1, *nk1;
    float2 *cand_stats;       // per candidate work item: (max, sum N exp(x - max)) of its candidates
    int2 *slice_cnt;          // last level: kept (clusters, keys) per slice of candidates (see launch_cand_select)
    float2 *row_stat;         // last level: the rows' (maximum, T * D)
    sq::DecodePlan cand;      // work items of candidate fine clusters (chunks of KPC clusters)
};

HierWs carve_hier(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H;
    const size_t items = rows * sq::chunk_cap_for(sh->C);
    HierWs w{};
    w.logits1 = cv.take<float>(rows * sh->C);
    w.logits2 = cv.take<float>(rows * sh->C);
    w.cand_id = cv.take<int32_t>(rows * sh->C);
    w.nr1 = cv.take<int32_t>(rows);
    w.nk1 = cv.take<int32_t>(rows);
    w.cand_stats = cv.take<float2>(items);
    w.slice_cnt = cv.take<int2>(rows * sq::cand_slices_for(sh->C));
    w.row_stat = cv.take<float2>(rows);
    w.cand.rec_cap = sh->C;
    w.cand.L = sh->C;
    w.cand.item_cap = (int)items;
    w.cand.rec = cv.take<int4>(rows * sh->C);
    w.cand.hdr = cv.take<int2>(rows);
    w.cand.row_items = cv.take<int2>(rows);
    w.cand.total = cv.take<int>(2);
    w.cand.item = cv.take<int2>(items * sq::ITEM_STRIDE);
    return w;
}

// Second candidate work list, for lookups of more than two levels.
sq::DecodePlan carve_cand_plan(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H;
    const size_t items = rows * sq::chunk_cap_for(sh->C);
    sq::DecodePlan p{};
    p.rec_cap = sh->C;
    p.L = sh->C;
    p.item_cap = (int)items;
    p.rec = cv.take<int4>(rows * sh->C);
    p.hdr = cv.take<int2>(rows);
    p.row_items = cv.take<int2>(rows);
    p.total = cv.take<int>(2);
    p.item = cv.take<int2>(items * sq::ITEM_STRIDE);
    return p;
}

// Workspace of one K-means iteration: half norms of the centres and the per-part histograms of centre ids.
struct KmeansWs {
    float *hn;
    int32_t *hist;
};

KmeansWs carve_kmeans(Carver &cv, const sq_shape_t *sh)
{
    const size_t heads = (size_t)sh->B * sh->H;
    const int PL = sq::kmeans_part_len(sh->L);
    const size_t parts = (size_t)(sh->L + PL - 1) / PL;
    KmeansWs w{};
    w.hn = cv.take<float>(heads * sh->C);
    w.hist = cv.take<int32_t>(heads * parts * sh->C);
    return w;
}

// Workspace of a hierarchical decode step.  Calls of up to KI_MAX_ROWS query rows and at least two levels attend
// through a key-index list (`indexed`: plan, partials, user slots as in IndexStepWs); others through the work-list
// kernels (dec).
struct HierStepWs {
    HierWs hier;
    uint32_t *mask1;
    int32_t *n_ranges, *n_keys;
    bool indexed;
    DecodeWs dec;
    sq::KeyIndexPlan plan;
    float *partials;
    int user_slot_base, nuq;
};

bool hier_step_is_indexed(const sq_shape_t *sh) { return (long long)sh->B * sh->H <= sq::KI_MAX_ROWS; }

HierStepWs carve_hier_step(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H;
    HierStepWs w{};
    w.hier = carve_hier(cv, sh);
    w.mask1 = cv.take<uint32_t>(rows * ((sh->C + 31) / 32));
    w.n_ranges = cv.take<int32_t>(rows);
    w.n_keys = cv.take<int32_t>(rows);
    w.indexed = hier_step_is_indexed(sh);
    if (w.indexed) {
        w.nuq = sq::user_pieces_for(sh->U);
        w.user_slot_base = sq::KI_ATTN_GRID + (int)rows;
        w.plan.L = sh->L;
        w.plan.row_keys = cv.take<int32_t>(rows);
        w.plan.key_idx = cv.take<int32_t>(rows * sh->L);
        w.partials = cv.take<float>(sq::keyidx_partial_slots((int)rows, w.nuq) * sq::PART_STRIDE);
    }
    w.dec = carve_decode(cv, sh);                      // (also a one-level "hierarchy" of an indexed call)
    return w;
}

// The dense attention over the user keys as extra workgroups of the key-index partial kernel.
sq::UserAttn make_user_pieces(const sq_shape_t *sh, int G, const void *q, const void *K_user, const void *V_user,
                              float *partials, int user_slot_base, int nuq)
{
    sq::UserAttn ua{};
    if (sh->U <= 0) return ua;
    ua.q = static_cast<const _Float16 *>(q);
    ua.Ku = static_cast<const _Float16 *>(K_user);
    ua.Vu = static_cast<const _Float16 *>(V_user);
    ua.partials = partials;
    ua.rows = sh->B * sh->H * G;
    ua.U = sh->U;
    ua.G = G;
    ua.nuq = nuq;
    ua.slot_base = user_slot_base;
    ua.sm_scale = sh->sm_scale;
    return ua;
}

// Workspace of the shared-set prefill attention: records of the kept ranges and the list of kept key rows.
struct PrefillSharedWs {
    sq::DecodePlan plan;
    int32_t *key_idx;
};

PrefillSharedWs carve_prefill_shared(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H;
    PrefillSharedWs w{};
    w.plan.rec_cap = sh->C;
    w.plan.L = sh->L;
    w.plan.rec = cv.take<int4>(rows * sh->C);
    w.plan.hdr = cv.take<int2>(rows);
    w.key_idx = cv.take<int32_t>(rows * sh->L);
    return w;
}

// Workspace of the whole prefill steps.
struct PrefillStepWs {
    uint32_t *mask;
    int32_t *n_ranges, *n_keys, *key_cid, *blk_info;
};

PrefillStepWs carve_prefill_step(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H * sh->Lq;
    PrefillStepWs w{};
    w.mask = cv.take<uint32_t>(rows * ((sh->C + 31) / 32));
    w.n_ranges = cv.take<int32_t>(rows);
    w.n_keys = cv.take<int32_t>(rows);
    w.key_cid = cv.take<int32_t>((size_t)sh->H * sh->L);
    w.blk_info = cv.take<int32_t>(sq::prefill_blk_info_ints(sh->H, sh->L));
    return w;
}

struct PrefillMeanStepWs {
    float *part_sum;
    int32_t *n_ranges, *n_keys;
    PrefillSharedWs att;
};

PrefillMeanStepWs carve_prefill_mean_step(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H;
    PrefillMeanStepWs w{};
    w.part_sum = cv.take<float>(rows * sq::lookup_parts_for(sh->Lq) * sh->C);
    w.n_ranges = cv.take<int32_t>(rows);
    w.n_keys = cv.take<int32_t>(rows);
    w.att = carve_prefill_shared(cv, sh);
    return w;
}

// Workspace of the hierarchical prefill step with per-query selection: the one-level step's, plus the level-1 masks
// and counts per token and the parent of every fine cluster.
struct HierPrefillWs {
    PrefillStepWs step;
    uint32_t *mask1;
    int32_t *nr1, *nk1, *parent;
};

HierPrefillWs carve_hier_prefill(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H * sh->Lq;
    HierPrefillWs w{};
    w.step = carve_prefill_step(cv, sh);
    w.mask1 = cv.take<uint32_t>(rows * 32);                 // at most 1024 coarse clusters
    w.nr1 = cv.take<int32_t>(rows);
    w.nk1 = cv.take<int32_t>(rows);
    w.parent = cv.take<int32_t>((size_t)sh->H * sh->C);
    return w;
}

// Workspace of the hierarchical prefill step on averaged scores: the one-level step's, plus the records of the kept
// coarse clusters' child ranges and the candidate list they expand to.
struct HierPrefillMeanWs {
    PrefillMeanStepWs step;
    sq::DecodePlan cand;
    int32_t *cand_id, *nr1, *nk1;
};

HierPrefillMeanWs carve_hier_prefill_mean(Carver &cv, const sq_shape_t *sh)
{
    const size_t rows = (size_t)sh->B * sh->H;
    HierPrefillMeanWs w{};
    w.step = carve_prefill_mean_step(cv, sh);
    w.cand.rec_cap = sh->C;
    w.cand.L = sh->C;
    w.cand.rec = cv.take<int4>(rows * sh->C);
    w.cand.hdr = cv.take<int2>(rows);
    w.cand_id = cv.take<int32_t>(rows * sh->C);
    w.nr1 = cv.take<int32_t>(rows);
    w.nk1 = cv.take<int32_t>(rows);
    return w;
}

int check_ws(const char *fn, const sq_shape_t *sh, int which, void *ws, size_t ws_bytes)
{
    const size_t need = sq_workspace_bytes(sh, which);
    if (need == 0) return SQ_OK;
    if (!ws) return fail(SQ_ERR_WORKSPACE, "%s: workspace is NULL, %zu bytes needed", fn, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(SQ_ERR_WORKSPACE, "%s: workspace is not 256-byte aligned", fn);
    if (ws_bytes < need) return fail(SQ_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, ws_bytes, need);
    return SQ_OK;
}

sq::Shape to_shape(const sq_shape_t *sh)
{
    return sq::Shape{sh->B, sh->H, sh->L, sh->C, sh->Lq, sh->U, sh->sm_scale, sh->causal_user};
}

}  // namespace

extern "C" {

int sq_version(void) { return 100; }

const char *sq_last_error(void) { return g_err; }

size_t sq_workspace_bytes(const sq_shape_t *sh, int which)
{
    if (!sh || sh->B <= 0 || sh->H <= 0 || sh->L <= 0 || sh->C <= 0 || sh->Lq <= 0 || sh->U < 0) return 0;
    Carver cv(nullptr);
    switch (which) {
    case SQ_CALL_ATTN_DECODE:
        carve_decode(cv, sh);
        return cv.off;
    case SQ_CALL_DECODE_STEP:
        if (step_is_shared(sh)) carve_step_shared(cv, sh);
        else if (step_is_indexed(sh)) carve_step_index(cv, sh);
        else carve_step(cv, sh);
        return cv.off;
    case SQ_CALL_ATTN_PREFILL:
        cv.take<int32_t>((size_t)sh->H * sh->L);
        cv.take<int32_t>(sq::prefill_blk_info_ints(sh->H, sh->L));
        return cv.off;
    case SQ_CALL_SELECT_MEAN:
        cv.take<float>((size_t)sh->B * sh->H * sq::mean_parts_for(sh->Lq) * sh->C);
        return cv.off;
    case SQ_CALL_ATTN_PREFILL_SHARED:
        carve_prefill_shared(cv, sh);
        return cv.off;
    case SQ_CALL_PREFILL_STEP:
        carve_prefill_step(cv, sh);
        return cv.off;
    case SQ_CALL_GQA_DECODE_STEP: {                     // sized for the largest group (16 query heads per K/V head)
        carve_step_shared(cv, sh, sq::SG);
        Carver cv2(nullptr), cv3(nullptr);              // ... on any of the kernel families
        carve_step(cv2, sh, sq::SG);
        carve_step_index(cv3, sh, sq::SG);
        size_t n = cv.off > cv2.off ? cv.off : cv2.off;
        return n > cv3.off ? n : cv3.off;
    }
    case SQ_CALL_MULTILEVEL_SELECT:
        carve_hier(cv, sh);
        carve_cand_plan(cv, sh);
        return cv.off;
    case SQ_CALL_MULTILEVEL_DECODE_STEP:
        carve_hier_step(cv, sh);
        carve_cand_plan(cv, sh);
        return cv.off;
    case SQ_CALL_KMEANS_STEP:
        carve_kmeans(cv, sh);
        return cv.off;
    case SQ_CALL_HIER_PREFILL_STEP:
        carve_hier_prefill(cv, sh);
        return cv.off;
    case SQ_CALL_GQA_MEAN_DECODE_STEP:                // sized for the largest group
        carve_step_shared(cv, sh, sq::SG);
        return cv.off;
    case SQ_CALL_HIER_PREFILL_MEAN_STEP:
        carve_hier_prefill_mean(cv, sh);
        return cv.off;
    case SQ_CALL_CALIBRATE:
        cv.take<float>((size_t)sh->B * sh->H * sh->Lq * sh->C);
        return cv.off;
    case SQ_CALL_PREFILL_MEAN_STEP:
        carve_prefill_mean_step(cv, sh);
        return cv.off;
    case SQ_CALL_HIER_SELECT:
        carve_hier(cv, sh);
        return cv.off;
    case SQ_CALL_HIER_DECODE_STEP:
        carve_hier_step(cv, sh);
        return cv.off;
    default:
        return 0;
    }
}

int sq_centroid_score(const sq_shape_t *sh, const void *q, const void *centroids, const int32_t *sizes, float *logits,
                      float *row_max, float *denom, void *, size_t, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(logits);
    SQ_REQUIRE_PTR(row_max);
    SQ_REQUIRE_PTR(denom);
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SQ_HIP(sq::launch_score(q, centroids, logits, nullptr, sh->B, sh->H, sh->Lq, sh->C, sh->sm_scale, s));
    SQ_HIP(sq::launch_row_stats(logits, sizes, row_max, denom, sh->B * sh->H * sh->Lq, sh->H, sh->Lq, sh->C, s));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_select(const sq_shape_t *sh, const float *logits, const float *row_max, const float *denom, const float *thresh,
              const int32_t *sizes, const int32_t *offsets, uint32_t *keep_mask, int32_t *ranges, int32_t *n_ranges,
              int32_t *n_keys, void *, size_t, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(logits);
    SQ_REQUIRE_PTR(row_max);
    SQ_REQUIRE_PTR(denom);
    SQ_REQUIRE_PTR(thresh);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(keep_mask);
    SQ_OPTIONAL_PTR(ranges);
    SQ_REQUIRE_PTR(n_ranges);
    SQ_REQUIRE_PTR(n_keys);
    if (int rc = check_device(__func__)) return rc;
    sq::DecodePlan none{};
    SQ_HIP(sq::launch_select(logits, row_max, denom, true, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys,
                             none, false, 0, sq::SelectOpts{}, sh->B * sh->H * sh->Lq, sh->H, sh->Lq, sh->C,
                             static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_sparse_attn_decode(const sq_shape_t *sh, const void *q, const void *K_fixed, const void *V_fixed,
                          const int32_t *ranges, const int32_t *n_ranges, const int32_t *n_keys, const void *K_user,
                          const void *V_user, void *out, float *lse, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    SQ_REQUIRE_PTR(ranges);
    SQ_REQUIRE_PTR(n_ranges);
    SQ_REQUIRE_PTR(n_keys);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    if (int rc = check_ws(__func__, sh, SQ_CALL_ATTN_DECODE, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    DecodeWs w = carve_decode(cv, sh);
    SQ_HIP(sq::launch_ranges_to_rec(ranges, n_ranges, w.plan, sh->B * sh->H, sh->C, s));
    SQ_HIP(sq::launch_schedule(w.plan, sh->B * sh->H, sh->U, s));
    SQ_HIP(sq::launch_decode_attn(q, K_fixed, V_fixed, K_user, V_user, w.plan, w.partials, out, lse, to_shape(sh), s));
    g_err[0] = 0;
    return SQ_OK;
}

namespace {
// Decode step over K/V shared by several query rows: B sequences over one fixed context, times G query heads per
// K/V head.  Every (sequence, query head) selects on its own; the work items are built from the union of the
// selections of each group of 16 of them, so a cluster kept by several is streamed once.
int decode_step_shared(const sq_shape_t *sh, int G, const void *q, const void *centroids, const int32_t *sizes,
                       const int32_t *offsets, const float *thresh, const void *K_fixed, const void *V_fixed,
                       const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask,
                       int32_t *n_keys, Carver &cv, hipStream_t s)
{
    SharedStepWs w = carve_step_shared(cv, sh, G);
    uint32_t *mask = keep_mask ? keep_mask : w.mask;
    // the G query heads of a (sequence, K/V head) are G query rows of that head: logits [B, H, G, C]
    SQ_HIP(sq::launch_score(q, centroids, w.logits, w.plan.total, sh->B, sh->H, G, sh->C, sh->sm_scale, s));
    SQ_HIP(sq::launch_union_schedule(w.logits, thresh, sizes, offsets, mask, w.n_ranges, n_keys ? n_keys : w.n_keys,
                                     w.plan, sh->U, sh->B, G, sh->H, sh->C, s));
    sq::Shape shp = to_shape(sh);
    shp.Lq = G;
    SQ_HIP(sq::launch_decode_attn_shared(q, K_fixed, V_fixed, K_user, V_user, w.plan, w.partials, out, lse, shp, s));
    return SQ_OK;
}
}  // namespace

namespace {
// Decode step of rows that are handled one by one (few query rows per K/V head), through the key-index list:
// score -> selection + key-index lists -> partial results over equal shares of the kept keys (the user keys in extra
// workgroups of the same launch) -> merge.  rows = B * H * G query rows [B, H, G]; K/V head of a row = (row / G) % H.
int decode_step_indexed(const sq_shape_t *sh, int G, const void *q, const void *centroids, const int32_t *sizes,
                        const int32_t *offsets, const float *thresh, const void *K_fixed, const void *V_fixed,
                        const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask,
                        int32_t *n_keys, Carver &cv, hipStream_t s)
{
    IndexStepWs w = carve_step_index(cv, sh, G);
    const int rows = sh->B * sh->H * G;
    const sq::UserAttn ua = make_user_pieces(sh, G, q, K_user, V_user, w.partials, w.user_slot_base, w.nuq);
    SQ_HIP(sq::launch_score(q, centroids, w.logits, nullptr, sh->B, sh->H, G, sh->C, sh->sm_scale, s));
    SQ_HIP(sq::launch_select_index(w.logits, thresh, sizes, offsets, keep_mask, w.n_ranges, n_keys ? n_keys : w.n_keys,
                                   w.plan, rows, sh->H, G, sh->C, s));
    SQ_HIP(sq::launch_decode_attn_index(q, K_fixed, V_fixed, w.plan, w.partials, out, lse, rows, sh->H, G, sh->sm_scale,
                                        &ua, s));
    return SQ_OK;
}
}  // namespace

int sq_gqa_decode_step(const sq_shape_t *sh, int32_t G, const void *q, const void *centroids, const int32_t *sizes,
                       const int32_t *offsets, const float *thresh, const void *K_fixed, const void *V_fixed,
                       const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask,
                       int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    if (G < 1 || G > sq::SG)
        return fail(SQ_ERR_UNSUPPORTED, "%s: G = %d query heads per K/V head; supported: 1 .. %d", __func__, G, sq::SG);
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(thresh);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_GQA_DECODE_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The shared-context kernels handle groups of 16 query rows and need the G rows of a sequence inside one group:
    // group sizes that do not divide 16 (3 or 6 query heads per K/V head) take the per-row kernels at any batch.
    if (step_is_shared(sh, G) && sq::SG % G == 0) {
        if (int rc = decode_step_shared(sh, G, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out,
                                        lse, keep_mask, n_keys, cv, s))
            return rc;
        g_err[0] = 0;
        return SQ_OK;
    }
    // Few query rows per K/V head: every (sequence, query head) is a row of the per-row kernels, which read the K/V
    // head once per query head (the rows are [B, H, G]: K/V head = (row / G) % H).
    if (step_is_indexed(sh, G)) {
        if (int rc = decode_step_indexed(sh, G, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out,
                                         lse, keep_mask, n_keys, cv, s))
            return rc;
        g_err[0] = 0;
        return SQ_OK;
    }
    StepWs w = carve_step(cv, sh, G);
    int32_t *nk = n_keys ? n_keys : w.n_keys;
    const int rows = sh->B * sh->H * G;
    SQ_HIP(sq::launch_score(q, centroids, w.logits, w.dec.plan.total, sh->B, sh->H, G, sh->C, sh->sm_scale, s));
    const sq::UserAttn ua = make_user_rider(sh, G, q, K_user, V_user, w.dec);
    SQ_HIP(sq::launch_select(w.logits, nullptr, nullptr, false, thresh, sizes, offsets, keep_mask, nullptr, w.n_ranges,
                             nk, w.dec.plan, true, ua.q ? 0 : sh->U, sq::SelectOpts{}, rows, sh->H, G, sh->C, s, &ua));
    sq::Shape shp = to_shape(sh);
    shp.Lq = G;
    SQ_HIP(sq::launch_decode_attn(q, K_fixed, V_fixed, K_user, V_user, w.dec.plan, w.dec.partials, out, lse, shp, s,
                                  ua.q ? ua.slot_base : -1, ua.nuq));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_gqa_mean_decode_step(const sq_shape_t *sh, int32_t G, const void *q, const void *centroids,
                            const int32_t *sizes, const int32_t *offsets, const float *thresh, const void *K_fixed,
                            const void *V_fixed, const void *K_user, const void *V_user, void *out, float *lse,
                            uint32_t *keep_mask, int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16)
        return fail(SQ_ERR_UNSUPPORTED, "%s: G = %d query heads per K/V head; supported: 1, 2, 4, 8, 16", __func__, G);
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(thresh);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_GQA_MEAN_DECODE_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    SharedStepWs w = carve_step_shared(cv, sh, G);
    SQ_HIP(sq::launch_score(q, centroids, w.logits, w.plan.total, sh->B, sh->H, G, sh->C, sh->sm_scale, s));
    SQ_HIP(sq::launch_group_mean_logits(w.logits, sizes, sh->B * sh->H, sh->H, G, sh->C, s));
    // The G rows of a group now select the same clusters: the union of a group of 16 rows streams each kept key once.
    SQ_HIP(sq::launch_union_schedule(w.logits, thresh, sizes, offsets, keep_mask ? keep_mask : w.mask, w.n_ranges,
                                     n_keys ? n_keys : w.n_keys, w.plan, sh->U, sh->B, G, sh->H, sh->C, s));
    sq::Shape shp = to_shape(sh);
    shp.Lq = G;
    SQ_HIP(sq::launch_decode_attn_shared(q, K_fixed, V_fixed, K_user, V_user, w.plan, w.partials, out, lse, shp, s));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_decode_step(const sq_shape_t *sh, const void *q, const void *centroids, const int32_t *sizes,
                   const int32_t *offsets, const float *thresh, const void *K_fixed, const void *V_fixed,
                   const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                   void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(thresh);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_DECODE_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    const int rows = sh->B * sh->H;
    if (step_is_shared(sh)) {
        if (int rc = decode_step_shared(sh, 1, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user,
                                        out, lse, keep_mask, n_keys, cv, s))
            return rc;
        g_err[0] = 0;
        return SQ_OK;
    }
    if (step_is_indexed(sh)) {
        if (int rc = decode_step_indexed(sh, 1, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out,
                                         lse, keep_mask, n_keys, cv, s))
            return rc;
        g_err[0] = 0;
        return SQ_OK;
    }
    StepWs w = carve_step(cv, sh);
    int32_t *nk = n_keys ? n_keys : w.n_keys;
    SQ_HIP(sq::launch_score(q, centroids, w.logits, w.dec.plan.total, sh->B, sh->H, 1, sh->C, sh->sm_scale, s));
    const sq::UserAttn ua = make_user_rider(sh, 1, q, K_user, V_user, w.dec);
    SQ_HIP(sq::launch_select(w.logits, nullptr, nullptr, false, thresh, sizes, offsets, keep_mask, nullptr, w.n_ranges,
                             nk, w.dec.plan, true, ua.q ? 0 : sh->U, sq::SelectOpts{}, rows, sh->H, 1, sh->C, s, &ua));
    SQ_HIP(sq::launch_decode_attn(q, K_fixed, V_fixed, K_user, V_user, w.dec.plan, w.dec.partials, out, lse,
                                  to_shape(sh), s, ua.q ? ua.slot_base : -1, ua.nuq));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_sparse_attn_prefill(const sq_shape_t *sh, const void *q, const void *K_fixed, const void *V_fixed,
                           const int32_t *offsets, const uint32_t *keep_mask, const void *K_user, const void *V_user,
                           void *out, float *lse, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(keep_mask);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    if (int rc = check_ws(__func__, sh, SQ_CALL_ATTN_PREFILL, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    int32_t *key_cid = cv.take<int32_t>((size_t)sh->H * sh->L);
    int32_t *blk_info = cv.take<int32_t>(sq::prefill_blk_info_ints(sh->H, sh->L));
    SQ_HIP(sq::launch_prefill_attn(q, K_fixed, V_fixed, K_user, V_user, keep_mask, offsets, key_cid, blk_info, out, lse,
                                   to_shape(sh), static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_select_mean(const sq_shape_t *sh, const float *logits, const float *row_max, const float *denom,
                   const float *thresh, const int32_t *sizes, const int32_t *offsets, uint32_t *keep_mask,
                   int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(logits);
    SQ_REQUIRE_PTR(row_max);
    SQ_REQUIRE_PTR(denom);
    SQ_REQUIRE_PTR(thresh);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(keep_mask);
    SQ_OPTIONAL_PTR(ranges);
    SQ_REQUIRE_PTR(n_ranges);
    SQ_REQUIRE_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_SELECT_MEAN, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    const int rows = sh->B * sh->H;
    float *part_sum = cv.take<float>((size_t)rows * sq::mean_parts_for(sh->Lq) * sh->C);
    SQ_HIP(sq::launch_mean_score(logits, row_max, denom, part_sum, rows, sh->Lq, sh->C, s));
    sq::SelectOpts opt{};
    opt.mean_parts = sq::mean_parts_for(sh->Lq);
    opt.mean_div = (float)sh->Lq;
    SQ_HIP(sq::launch_select(part_sum, nullptr, nullptr, true, thresh, sizes, offsets, keep_mask, ranges, n_ranges,
                             n_keys, sq::DecodePlan{}, false, 0, opt, rows, sh->H, 1, sh->C, s));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_sparse_attn_prefill_shared(const sq_shape_t *sh, const void *q, const void *K_fixed, const void *V_fixed,
                                  const int32_t *ranges, const int32_t *n_ranges, const int32_t *n_keys,
                                  const void *K_user, const void *V_user, void *out, float *lse, void *ws,
                                  size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    SQ_REQUIRE_PTR(ranges);
    SQ_REQUIRE_PTR(n_ranges);
    SQ_REQUIRE_PTR(n_keys);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    if (int rc = check_ws(__func__, sh, SQ_CALL_ATTN_PREFILL_SHARED, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    PrefillSharedWs w = carve_prefill_shared(cv, sh);
    SQ_HIP(sq::launch_ranges_to_rec(ranges, n_ranges, w.plan, sh->B * sh->H, sh->C, s));
    SQ_HIP(sq::launch_prefill_attn_shared(q, K_fixed, V_fixed, K_user, V_user, w.plan, w.key_idx, out, lse,
                                          to_shape(sh), s));
    g_err[0] = 0;
    return SQ_OK;
}

// Pointer checks shared by the two whole prefill steps (same argument list).
#define SQ_PREFILL_STEP_PTRS()      \
    SQ_REQUIRE_PTR(q);              \
    SQ_REQUIRE_PTR(centroids);      \
    SQ_REQUIRE_PTR(sizes);          \
    SQ_REQUIRE_PTR(offsets);        \
    SQ_REQUIRE_PTR(thresh);         \
    SQ_REQUIRE_PTR(K_fixed);        \
    SQ_REQUIRE_PTR(V_fixed);        \
    if (sh->U > 0) {                \
        SQ_REQUIRE_PTR(K_user);     \
        SQ_REQUIRE_PTR(V_user);     \
    }                               \
    SQ_REQUIRE_PTR(out);            \
    SQ_OPTIONAL_PTR(lse);           \
    SQ_OPTIONAL_PTR(keep_mask);     \
    SQ_OPTIONAL_PTR(n_keys)

int sq_prefill_step(const sq_shape_t *sh, const void *q, const void *centroids, const int32_t *sizes,
                    const int32_t *offsets, const float *thresh, const void *K_fixed, const void *V_fixed,
                    const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                    void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_PREFILL_STEP_PTRS();
    if (int rc = check_ws(__func__, sh, SQ_CALL_PREFILL_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    PrefillStepWs w = carve_prefill_step(cv, sh);
    uint32_t *mask = keep_mask ? keep_mask : w.mask;
    SQ_HIP(sq::launch_prefill_lookup(q, centroids, sizes, thresh, mask, w.n_ranges, n_keys ? n_keys : w.n_keys, nullptr,
                                     false, sh->B, sh->H, sh->Lq, sh->C, sh->sm_scale, s));
    SQ_HIP(sq::launch_prefill_attn(q, K_fixed, V_fixed, K_user, V_user, mask, offsets, w.key_cid, w.blk_info, out, lse,
                                   to_shape(sh), s));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_prefill_mean_step(const sq_shape_t *sh, const void *q, const void *centroids, const int32_t *sizes,
                         const int32_t *offsets, const float *thresh, const void *K_fixed, const void *V_fixed,
                         const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask,
                         int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_PREFILL_STEP_PTRS();
    if (int rc = check_ws(__func__, sh, SQ_CALL_PREFILL_MEAN_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    PrefillMeanStepWs w = carve_prefill_mean_step(cv, sh);
    const int rows = sh->B * sh->H;
    SQ_HIP(sq::launch_prefill_lookup(q, centroids, sizes, thresh, nullptr, nullptr, nullptr, w.part_sum, true, sh->B,
                                     sh->H, sh->Lq, sh->C, sh->sm_scale, s));
    sq::SelectOpts opt{};
    opt.mean_parts = sq::lookup_parts_for(sh->Lq);
    opt.mean_div = (float)sh->Lq;
    // the selection writes the kept ranges' records straight into the attention's plan
    SQ_HIP(sq::launch_select(w.part_sum, nullptr, nullptr, true, thresh, sizes, offsets, keep_mask, nullptr, w.n_ranges,
                             n_keys ? n_keys : w.n_keys, w.att.plan, false, 0, opt, rows, sh->H, 1, sh->C, s));
    SQ_HIP(sq::launch_prefill_attn_shared(q, K_fixed, V_fixed, K_user, V_user, w.att.plan, w.att.key_idx, out, lse,
                                          to_shape(sh), s));
    g_err[0] = 0;
    return SQ_OK;
}

namespace {

// Both levels of the lookup (Section 3.3).  plan2 (may be empty) receives the level-2 records and, when
// `schedule2`, the attention work items.
// One level of a centroid hierarchy as the lookup sees it (mask: optional output of the level).
struct Level {
    int C;
    const void *centroids;
    const int32_t *sizes, *child_offsets;
    const float *thresh;
    uint32_t *mask;
};

// Lookup through n >= 1 levels, coarsest first (Section 3.3, Eq. 2 then Eq. 3 level after level).  Level 0 scores
// all of its clusters; a kept cluster's child range becomes chunks of candidate clusters of the next level (a
// balanced number of centroids per workgroup, Appendix D); every further level scores its candidates only
// (logits in candidate order) and selects over that list, so its maximum and normaliser run over the candidates
// only.  The candidate work lists of consecutive levels alternate between w.cand and cand_b (a level reads one
// while it fills the other).  The last level writes ranges / counts and, when `schedule_last`, the attention
// work items into plan_last.  klast (n >= 2): the last level is selected in slices of its candidates, many workgroups
// per row (launch_cand_select), and leaves the rows' key-index lists in *klast instead of work items (decode steps of at
// most KI_MAX_ROWS rows; the lookup alone keeps one workgroup per row).
int multilevel_lookup(const char *fn, const sq_shape_t *sh, int n, const Level *lv, const void *q, int32_t *ranges,
                      int32_t *n_ranges, int32_t *n_keys, HierWs &w, sq::DecodePlan cand_b, sq::DecodePlan plan_last,
                      bool schedule_last, hipStream_t s, const sq::UserAttn *user = nullptr,
                      const sq::KeyIndexPlan *klast = nullptr)
{
    // `user` (decode steps): the rows' user-key attention rides on the level-0 selection launch (see
    // make_user_rider), and the attention work list of the last level then holds no user chunks.
    const bool rider = user && user->q;
    const int U_last = rider ? 0 : sh->U;
    const int rows = sh->B * sh->H;
    hipError_t e;
    if (n == 1) {
        e = sq::launch_score(q, lv[0].centroids, w.logits1, plan_last.total, sh->B, sh->H, 1, lv[0].C, sh->sm_scale, s);
        if (e == hipSuccess)
            e = sq::launch_select(w.logits1, nullptr, nullptr, false, lv[0].thresh, lv[0].sizes, lv[0].child_offsets,
                                  lv[0].mask, ranges, n_ranges, n_keys, plan_last, schedule_last, U_last, sq::SelectOpts{},
                                  rows, sh->H, 1, lv[0].C, s, user);
        if (e != hipSuccess) return fail(SQ_ERR_HIP, "%s: launch failed -> %s", fn, hipGetErrorString(e));
        return SQ_OK;
    }
    sq::DecodePlan cur = w.cand, nxt = cand_b;
    e = sq::launch_score(q, lv[0].centroids, w.logits1, cur.total, sh->B, sh->H, 1, lv[0].C, sh->sm_scale, s);
    if (e == hipSuccess) {
        sq::SelectOpts o{};
        o.len_from_offsets = 1;
        cur.rec_cap = lv[0].C;
        e = sq::launch_select(w.logits1, nullptr, nullptr, false, lv[0].thresh, lv[0].sizes, lv[0].child_offsets,
                              lv[0].mask, nullptr, w.nr1, w.nk1, cur, true, 0, o, rows, sh->H, 1, lv[0].C, s, user);
    }
    for (int k = 1; k < n && e == hipSuccess; ++k) {
        const bool last = k == n - 1;
        sq::DecodePlan dst = last ? plan_last : nxt;
        // (the records of `cur` were consumed when its work items were written: the array now takes the candidates')
        const bool sliced = last && klast;
        e = sq::launch_gather_score(q, lv[k].centroids, cur, lv[k].sizes, lv[k].child_offsets, last ? 0 : 1, w.logits2,
                                    w.cand_id, cur.rec, w.cand_stats, sliced ? nullptr : dst.total, sh->H, lv[k].C,
                                    sh->sm_scale, s, sliced ? lv[k].mask : nullptr,
                                    (size_t)rows * ((lv[k].C + 31) / 32));
        if (e != hipSuccess) break;
        if (sliced) {
            const sq::CandSelect cs{cur.rec, cur.hdr, w.cand_stats, cur.row_items, w.slice_cnt, w.row_stat};
            e = sq::launch_cand_select(cs, lv[k].thresh, lv[k].mask, n_ranges, n_keys, *klast, rows, sh->H, lv[k].C, s);
            break;
        }
        sq::SelectOpts o{};
        o.cand_id = w.cand_id;
        o.cand_hdr = cur.hdr;
        o.cand_rec = cur.rec;
        o.cand_stats = w.cand_stats;
        o.cand_items = cur.row_items;
        if (last) {
            e = sq::launch_select(w.logits2, nullptr, nullptr, false, lv[k].thresh, lv[k].sizes, lv[k].child_offsets,
                                  lv[k].mask, ranges, n_ranges, n_keys, plan_last, schedule_last, U_last, o, rows, sh->H, 1,
                                  lv[k].C, s);
        } else {
            o.len_from_offsets = 1;
            dst.rec_cap = lv[k].C;
            e = sq::launch_select(w.logits2, nullptr, nullptr, false, lv[k].thresh, lv[k].sizes, lv[k].child_offsets,
                                  lv[k].mask, nullptr, w.nr1, w.nk1, dst, true, 0, o, rows, sh->H, 1, lv[k].C, s);
            nxt = cur;
            cur = dst;
        }
    }
    if (e != hipSuccess) return fail(SQ_ERR_HIP, "%s: launch failed -> %s", fn, hipGetErrorString(e));
    return SQ_OK;
}

int hier_lookup(const char *fn, const sq_shape_t *sh, int32_t C1, const void *q, const void *centroids1,
                const int32_t *sizes1, const int32_t *child_offsets, const float *thresh1, const void *centroids2,
                const int32_t *sizes2, const int32_t *offsets2, const float *thresh2, uint32_t *keep_mask1,
                uint32_t *keep_mask2, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, HierWs &w,
                sq::DecodePlan plan2, bool schedule2, hipStream_t s, const sq::UserAttn *user = nullptr,
                const sq::KeyIndexPlan *klast = nullptr)
{
    const Level lv[2] = {{C1, centroids1, sizes1, child_offsets, thresh1, keep_mask1},
                         {sh->C, centroids2, sizes2, offsets2, thresh2, keep_mask2}};
    return multilevel_lookup(fn, sh, 2, lv, q, ranges, n_ranges, n_keys, w, sq::DecodePlan{}, plan2, schedule2, s, user,
                             klast);
}

// Validates a caller's level array and copies it (masks: optional host array of per-level outputs).
int read_levels(const char *fn, const sq_shape_t *sh, int32_t n, const sq_level_t *levels, uint32_t *const *masks,
                Level *lv)
{
    if (n < 1 || n > SQ_MAX_LEVELS) return fail(SQ_ERR_INVALID_ARG, "%s: n_levels = %d must be in [1, %d]", fn, n, SQ_MAX_LEVELS);
    if (!levels) return fail(SQ_ERR_INVALID_ARG, "%s: levels is NULL", fn);
    for (int k = 0; k < n; ++k) {
        const sq_level_t &l = levels[k];
        if (l.C <= 0 || l.C > sh->C)
            return fail(SQ_ERR_INVALID_ARG, "%s: levels[%d].C = %d must be in [1, shape->C = %d]", fn, k, l.C, sh->C);
        const void *ptrs[4] = {l.centroids, l.sizes, l.child_offsets, l.thresh};
        for (const void *p : ptrs)
            if (!p || !aligned16(p)) return fail(SQ_ERR_INVALID_ARG, "%s: a pointer of levels[%d] is NULL or not 16-byte aligned", fn, k);
        uint32_t *m = masks ? masks[k] : nullptr;
        if (m && !aligned16(m)) return fail(SQ_ERR_INVALID_ARG, "%s: keep_masks[%d] is not 16-byte aligned", fn, k);
        lv[k] = Level{l.C, l.centroids, l.sizes, l.child_offsets, l.thresh, m};
    }
    if (levels[n - 1].C != sh->C)
        return fail(SQ_ERR_INVALID_ARG, "%s: the last level has %d clusters, shape->C is %d", fn, levels[n - 1].C, sh->C);
    return SQ_OK;
}

int check_hier_args(const char *fn, const sq_shape_t *sh, int32_t C1)
{
    if (C1 <= 0 || C1 > sh->C) return fail(SQ_ERR_INVALID_ARG, "%s: C1 = %d must be in [1, C2 = %d]", fn, C1, sh->C);
    return SQ_OK;
}

}  // namespace

int sq_hier_select(const sq_shape_t *sh, int32_t C1, const void *q, const void *centroids1, const int32_t *sizes1,
                   const int32_t *child_offsets, const float *thresh1, const void *centroids2, const int32_t *sizes2,
                   const int32_t *offsets2, const float *thresh2, uint32_t *keep_mask1, uint32_t *keep_mask2,
                   int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    if (int rc = check_hier_args(__func__, sh, C1)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids1);
    SQ_REQUIRE_PTR(sizes1);
    SQ_REQUIRE_PTR(child_offsets);
    SQ_REQUIRE_PTR(thresh1);
    SQ_REQUIRE_PTR(centroids2);
    SQ_REQUIRE_PTR(sizes2);
    SQ_REQUIRE_PTR(offsets2);
    SQ_REQUIRE_PTR(thresh2);
    SQ_REQUIRE_PTR(keep_mask1);
    SQ_REQUIRE_PTR(keep_mask2);
    SQ_OPTIONAL_PTR(ranges);
    SQ_REQUIRE_PTR(n_ranges);
    SQ_REQUIRE_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_HIER_SELECT, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    HierWs w = carve_hier(cv, sh);
    if (int rc = hier_lookup(__func__, sh, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2,
                             offsets2, thresh2, keep_mask1, keep_mask2, ranges, n_ranges, n_keys, w, sq::DecodePlan{},
                             false, static_cast<hipStream_t>(stream)))
        return rc;
    g_err[0] = 0;
    return SQ_OK;
}

int sq_hier_decode_step(const sq_shape_t *sh, int32_t C1, const void *q, const void *centroids1,
                        const int32_t *sizes1, const int32_t *child_offsets, const float *thresh1,
                        const void *centroids2, const int32_t *sizes2, const int32_t *offsets2, const float *thresh2,
                        const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user, void *out,
                        float *lse, uint32_t *keep_mask2, int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    if (int rc = check_hier_args(__func__, sh, C1)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids1);
    SQ_REQUIRE_PTR(sizes1);
    SQ_REQUIRE_PTR(child_offsets);
    SQ_REQUIRE_PTR(thresh1);
    SQ_REQUIRE_PTR(centroids2);
    SQ_REQUIRE_PTR(sizes2);
    SQ_REQUIRE_PTR(offsets2);
    SQ_REQUIRE_PTR(thresh2);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask2);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_HIER_DECODE_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    HierStepWs w = carve_hier_step(cv, sh);
    if (w.indexed) {
        if (int rc = hier_lookup(__func__, sh, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2,
                                 offsets2, thresh2, w.mask1, keep_mask2, nullptr, w.n_ranges, n_keys ? n_keys : w.n_keys,
                                 w.hier, sq::DecodePlan{}, false, s, nullptr, &w.plan))
            return rc;
        const sq::UserAttn ua = make_user_pieces(sh, 1, q, K_user, V_user, w.partials, w.user_slot_base, w.nuq);
        SQ_HIP(sq::launch_decode_attn_index(q, K_fixed, V_fixed, w.plan, w.partials, out, lse, sh->B * sh->H, sh->H, 1,
                                            sh->sm_scale, &ua, s));
        g_err[0] = 0;
        return SQ_OK;
    }
    const sq::UserAttn ua = make_user_rider(sh, 1, q, K_user, V_user, w.dec);
    if (int rc = hier_lookup(__func__, sh, C1, q, centroids1, sizes1, child_offsets, thresh1, centroids2, sizes2,
                             offsets2, thresh2, w.mask1, keep_mask2, nullptr, w.n_ranges, n_keys ? n_keys : w.n_keys,
                             w.hier, w.dec.plan, true, s, &ua))
        return rc;
    SQ_HIP(sq::launch_decode_attn(q, K_fixed, V_fixed, K_user, V_user, w.dec.plan, w.dec.partials, out, lse,
                                  to_shape(sh), s, ua.q ? ua.slot_base : -1, ua.nuq));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_hier_prefill_step(const sq_shape_t *sh, int32_t C1, const void *q, const void *centroids1, const int32_t *sizes1,
                         const int32_t *child_offsets, const float *thresh1, const void *centroids2,
                         const int32_t *sizes2, const int32_t *offsets2, const float *thresh2, const void *K_fixed,
                         const void *V_fixed, const void *K_user, const void *V_user, void *out, float *lse,
                         uint32_t *keep_mask2, int32_t *n_keys, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    if (int rc = check_hier_args(__func__, sh, C1)) return rc;
    if (C1 > 1024)
        return fail(SQ_ERR_UNSUPPORTED, "%s: C1 = %d coarse clusters; per-query prefill supports at most 1024", __func__, C1);
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids1);
    SQ_REQUIRE_PTR(sizes1);
    SQ_REQUIRE_PTR(child_offsets);
    SQ_REQUIRE_PTR(thresh1);
    SQ_REQUIRE_PTR(centroids2);
    SQ_REQUIRE_PTR(sizes2);
    SQ_REQUIRE_PTR(offsets2);
    SQ_REQUIRE_PTR(thresh2);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask2);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_HIER_PREFILL_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    HierPrefillWs w = carve_hier_prefill(cv, sh);
    uint32_t *mask2 = keep_mask2 ? keep_mask2 : w.step.mask;
    // Level 1 (Eq. 2) per token over the coarse centroids; then every fine cluster's parent; then level 2 (Eq. 3) per
    // token over the children of the coarse clusters that token kept.
    SQ_HIP(sq::launch_prefill_lookup(q, centroids1, sizes1, thresh1, w.mask1, w.nr1, w.nk1, nullptr, false, sh->B, sh->H,
                                     sh->Lq, C1, sh->sm_scale, s));
    SQ_HIP(sq::launch_child_parent(child_offsets, w.parent, sh->H, C1, sh->C, s));
    SQ_HIP(sq::launch_prefill_lookup(q, centroids2, sizes2, thresh2, mask2, w.step.n_ranges,
                                     n_keys ? n_keys : w.step.n_keys, nullptr, false, sh->B, sh->H, sh->Lq, sh->C,
                                     sh->sm_scale, s, nullptr, nullptr, w.parent, w.mask1, C1));
    SQ_HIP(sq::launch_prefill_attn(q, K_fixed, V_fixed, K_user, V_user, mask2, offsets2, w.step.key_cid, w.step.blk_info,
                                   out, lse, to_shape(sh), s));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_hier_prefill_mean_step(const sq_shape_t *sh, int32_t C1, const void *q, const void *centroids1,
                              const int32_t *sizes1, const int32_t *child_offsets, const float *thresh1,
                              const void *centroids2, const int32_t *sizes2, const int32_t *offsets2,
                              const float *thresh2, const void *K_fixed, const void *V_fixed, const void *K_user,
                              const void *V_user, void *out, float *lse, uint32_t *keep_mask2, int32_t *n_keys, void *ws,
                              size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    if (int rc = check_hier_args(__func__, sh, C1)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(centroids1);
    SQ_REQUIRE_PTR(sizes1);
    SQ_REQUIRE_PTR(child_offsets);
    SQ_REQUIRE_PTR(thresh1);
    SQ_REQUIRE_PTR(centroids2);
    SQ_REQUIRE_PTR(sizes2);
    SQ_REQUIRE_PTR(offsets2);
    SQ_REQUIRE_PTR(thresh2);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask2);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_HIER_PREFILL_MEAN_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    HierPrefillMeanWs w = carve_hier_prefill_mean(cv, sh);
    const int rows = sh->B * sh->H;
    sq::SelectOpts opt{};
    opt.mean_parts = sq::lookup_parts_for(sh->Lq);
    opt.mean_div = (float)sh->Lq;
    // Level 1 (Eq. 2 averaged over the tokens): the kept coarse clusters' child ranges become records ...
    SQ_HIP(sq::launch_prefill_lookup(q, centroids1, sizes1, thresh1, nullptr, nullptr, nullptr, w.step.part_sum, true,
                                     sh->B, sh->H, sh->Lq, C1, sh->sm_scale, s));
    sq::SelectOpts opt1 = opt;
    opt1.len_from_offsets = 1;
    SQ_HIP(sq::launch_select(w.step.part_sum, nullptr, nullptr, true, thresh1, sizes1, child_offsets, nullptr, nullptr,
                             w.nr1, w.nk1, w.cand, false, 0, opt1, rows, sh->H, 1, C1, s));
    // ... which expand to the list of candidate fine clusters of each (sequence, head).
    SQ_HIP(sq::launch_expand_ranges(w.cand, w.cand_id, rows, sh->C, s));
    // Level 2 (Eq. 3 per token over the candidates, averaged over the tokens): scores and selection in candidate order.
    SQ_HIP(sq::launch_prefill_lookup(q, centroids2, sizes2, thresh2, nullptr, nullptr, nullptr, w.step.part_sum, true,
                                     sh->B, sh->H, sh->Lq, sh->C, sh->sm_scale, s, w.cand_id, w.cand.hdr));
    sq::SelectOpts opt2 = opt;
    opt2.cand_id = w.cand_id;
    opt2.cand_hdr = w.cand.hdr;
    SQ_HIP(sq::launch_select(w.step.part_sum, nullptr, nullptr, true, thresh2, sizes2, offsets2, keep_mask2, nullptr,
                             w.step.n_ranges, n_keys ? n_keys : w.step.n_keys, w.step.att.plan, false, 0, opt2, rows,
                             sh->H, 1, sh->C, s));
    SQ_HIP(sq::launch_prefill_attn_shared(q, K_fixed, V_fixed, K_user, V_user, w.step.att.plan, w.step.att.key_idx, out,
                                          lse, to_shape(sh), s));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_multilevel_select(const sq_shape_t *sh, int32_t n_levels, const sq_level_t *levels, const void *q,
                         uint32_t *const *keep_masks, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, void *ws,
                         size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    Level lv[SQ_MAX_LEVELS];
    if (int rc = read_levels(__func__, sh, n_levels, levels, keep_masks, lv)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_OPTIONAL_PTR(ranges);
    SQ_REQUIRE_PTR(n_ranges);
    SQ_REQUIRE_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_MULTILEVEL_SELECT, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    HierWs w = carve_hier(cv, sh);
    sq::DecodePlan cand_b = carve_cand_plan(cv, sh);
    if (int rc = multilevel_lookup(__func__, sh, n_levels, lv, q, ranges, n_ranges, n_keys, w, cand_b, sq::DecodePlan{},
                                   false, static_cast<hipStream_t>(stream)))
        return rc;
    g_err[0] = 0;
    return SQ_OK;
}

int sq_multilevel_decode_step(const sq_shape_t *sh, int32_t n_levels, const sq_level_t *levels, const void *q,
                              const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                              void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys, void *ws, size_t ws_bytes,
                              void *stream)
{
    if (int rc = check_shape(sh, __func__, true)) return rc;
    Level lv[SQ_MAX_LEVELS];
    if (int rc = read_levels(__func__, sh, n_levels, levels, nullptr, lv)) return rc;
    SQ_REQUIRE_PTR(q);
    SQ_REQUIRE_PTR(K_fixed);
    SQ_REQUIRE_PTR(V_fixed);
    if (sh->U > 0) {
        SQ_REQUIRE_PTR(K_user);
        SQ_REQUIRE_PTR(V_user);
    }
    SQ_REQUIRE_PTR(out);
    SQ_OPTIONAL_PTR(lse);
    SQ_OPTIONAL_PTR(keep_mask);
    SQ_OPTIONAL_PTR(n_keys);
    if (int rc = check_ws(__func__, sh, SQ_CALL_MULTILEVEL_DECODE_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Carver cv(ws);
    HierStepWs w = carve_hier_step(cv, sh);
    sq::DecodePlan cand_b = carve_cand_plan(cv, sh);
    lv[n_levels - 1].mask = keep_mask;
    if (w.indexed && n_levels >= 2) {
        if (int rc = multilevel_lookup(__func__, sh, n_levels, lv, q, nullptr, w.n_ranges, n_keys ? n_keys : w.n_keys,
                                       w.hier, cand_b, sq::DecodePlan{}, false, s, nullptr, &w.plan))
            return rc;
        const sq::UserAttn ua = make_user_pieces(sh, 1, q, K_user, V_user, w.partials, w.user_slot_base, w.nuq);
        SQ_HIP(sq::launch_decode_attn_index(q, K_fixed, V_fixed, w.plan, w.partials, out, lse, sh->B * sh->H, sh->H, 1,
                                            sh->sm_scale, &ua, s));
        g_err[0] = 0;
        return SQ_OK;
    }
    const sq::UserAttn ua = make_user_rider(sh, 1, q, K_user, V_user, w.dec);
    if (int rc = multilevel_lookup(__func__, sh, n_levels, lv, q, nullptr, w.n_ranges, n_keys ? n_keys : w.n_keys, w.hier,
                                   cand_b, w.dec.plan, true, s, &ua))
        return rc;
    SQ_HIP(sq::launch_decode_attn(q, K_fixed, V_fixed, K_user, V_user, w.dec.plan, w.dec.partials, out, lse,
                                  to_shape(sh), s, ua.q ? ua.slot_base : -1, ua.nuq));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_kmeans_normalize(const sq_shape_t *sh, const void *K, void *X, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(K);
    SQ_REQUIRE_PTR(X);
    if (int rc = check_device(__func__)) return rc;
    SQ_HIP(sq::launch_normalize_rows(K, X, (size_t)sh->B * sh->H * sh->L, static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_kmeans_step(const sq_shape_t *sh, const void *X, const void *centers_in, void *centers_out, int32_t *assign,
                   int32_t *sizes, int32_t *offsets, int32_t *perm, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    if (sh->C > sh->L) return fail(SQ_ERR_INVALID_ARG, "%s: more centres (%d) than keys (%d)", __func__, sh->C, sh->L);
    SQ_REQUIRE_PTR(X);
    SQ_REQUIRE_PTR(centers_in);
    SQ_REQUIRE_PTR(centers_out);
    SQ_REQUIRE_PTR(assign);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(perm);
    if (int rc = check_ws(__func__, sh, SQ_CALL_KMEANS_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    KmeansWs w = carve_kmeans(cv, sh);
    SQ_HIP(sq::launch_kmeans_step(X, centers_in, centers_out, assign, sizes, offsets, perm, w.hn, w.hist, sh->B * sh->H,
                                  sh->L, sh->C, static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_cluster_layout(const sq_shape_t *sh, const void *K, const void *V, const int32_t *perm, const int32_t *sizes,
                      const int32_t *offsets, void *K_sorted, void *V_sorted, void *centroids, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    SQ_REQUIRE_PTR(K);
    SQ_OPTIONAL_PTR(V);
    SQ_OPTIONAL_PTR(perm);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_OPTIONAL_PTR(K_sorted);
    SQ_OPTIONAL_PTR(V_sorted);
    SQ_REQUIRE_PTR(centroids);
    if (V_sorted && (!V || !K_sorted))
        return fail(SQ_ERR_INVALID_ARG, "%s: V_sorted needs V and K_sorted", __func__);
    if (K_sorted && !perm) return fail(SQ_ERR_INVALID_ARG, "%s: reordering needs perm", __func__);
    if (K_sorted && (K_sorted == K || K_sorted == V || (V_sorted && (V_sorted == V || V_sorted == K))))
        return fail(SQ_ERR_INVALID_ARG, "%s: the reordered tensors must not alias the inputs", __func__);
    if (int rc = check_device(__func__)) return rc;
    SQ_HIP(sq::launch_cluster_layout(K, V, perm, sizes, offsets, K_sorted, V_sorted, centroids, sh->B * sh->H, sh->L,
                                     sh->C, static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_cluster_nest(const sq_shape_t *sh, int32_t C1, const int32_t *assign_fine, const int32_t *perm_coarse,
                    const int32_t *child_offsets, int32_t *assign_new, int32_t *sizes, int32_t *offsets, int32_t *perm,
                    int32_t *sizes_coarse, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    if (C1 <= 0 || C1 > sh->C) return fail(SQ_ERR_INVALID_ARG, "%s: C1 = %d must be in [1, C = %d]", __func__, C1, sh->C);
    SQ_REQUIRE_PTR(assign_fine);
    SQ_REQUIRE_PTR(perm_coarse);
    SQ_REQUIRE_PTR(child_offsets);
    SQ_REQUIRE_PTR(assign_new);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(offsets);
    SQ_REQUIRE_PTR(perm);
    SQ_REQUIRE_PTR(sizes_coarse);
    if (int rc = check_ws(__func__, sh, SQ_CALL_KMEANS_STEP, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    KmeansWs w = carve_kmeans(cv, sh);
    SQ_HIP(sq::launch_cluster_nest(assign_fine, perm_coarse, child_offsets, assign_new, sizes, offsets, perm, sizes_coarse,
                                   reinterpret_cast<int32_t *>(w.hn), w.hist, sh->B * sh->H, sh->L, sh->C, C1,
                                   static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

int sq_calibrate_threshold(const sq_shape_t *sh, const float *logits, const float *row_max, const float *denom,
                           const int32_t *sizes, int64_t target_keys, float *thresh, void *ws, size_t ws_bytes,
                           void *stream)
{
    if (int rc = check_shape(sh, __func__, false)) return rc;
    if (target_keys < 0) return fail(SQ_ERR_INVALID_ARG, "%s: target_keys is negative", __func__);
    if ((long long)sh->B * sh->Lq * sh->L >= (1ll << 31) || (long long)sh->B * sh->Lq * sh->C >= (1ll << 30))
        return fail(SQ_ERR_UNSUPPORTED, "%s: too many calibration queries (B * Lq * L must stay below 2^31)", __func__);
    SQ_REQUIRE_PTR(logits);
    SQ_REQUIRE_PTR(row_max);
    SQ_REQUIRE_PTR(denom);
    SQ_REQUIRE_PTR(sizes);
    SQ_REQUIRE_PTR(thresh);
    if (int rc = check_ws(__func__, sh, SQ_CALL_CALIBRATE, ws, ws_bytes)) return rc;
    if (int rc = check_device(__func__)) return rc;
    Carver cv(ws);
    float *S = cv.take<float>((size_t)sh->B * sh->H * sh->Lq * sh->C);
    const long long cap = (long long)sh->B * sh->Lq * sh->L;
    SQ_HIP(sq::launch_calibrate(logits, row_max, denom, sizes, S, thresh, (int)(target_keys < cap ? target_keys : cap),
                                sh->B, sh->H, sh->Lq, sh->C, static_cast<hipStream_t>(stream)));
    g_err[0] = 0;
    return SQ_OK;
}

}  // extern "C"
