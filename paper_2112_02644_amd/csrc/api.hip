// Host runtime behind the C ABI of include/smtm.h: context, device tables, argument checks,
// launch order.  Every entry point validates its arguments before it touches the GPU and only
// enqueues work on the caller's stream; the few calls that synchronise say so in the header.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "internal.h"

using namespace smtm;

struct smtm_ctx {
    smtm_config cfg;
    int device;
    char err[512];

    int n_pad;                                   // classes rounded up to kRowPad (fp16 operand rows, fast-memory mask)
    int Cp[SMTM_MAX_EXITS];                      // channels rounded up to kKPad
    int tiles;                                   // class tiles of the scoring kernels

    // global memory (Sec. 6): centres per exit point, update counts, tables
    float* centres[SMTM_MAX_EXITS];              // [n, C_l] fp32 master
    float* cinv[SMTM_MAX_EXITS];                 // [n] 1/|SC_j| (0 = degenerate)
    _Float16* chat[SMTM_MAX_EXITS];              // [n_pad, Cp_l] unit fp16 copy, zero padded
    uint32_t* mcount[SMTM_MAX_EXITS];            // [n]
    uint32_t* FT;
    uint32_t* TS;
    // fast memory
    int32_t* hot_ids;                            // [hot_max] policy order
    uint8_t* in_hot;                             // [n]
    int32_t* ids_stage;                          // [hot_max] staging for smtm_hot_set
    // batch state
    float* SA;                                   // [max_batch, n] by original frame id (+ slack for unguarded tile loads)
    float* sv[SMTM_MAX_EXITS];                   // [max_batch, Cp_l] by live slot at that exit point, columns >= C_l stay zero
    int32_t* slot_of[SMTM_MAX_EXITS];            // [max_batch] live slot each frame had at that exit point
    uint32_t* rowmax;                            // [L, max_batch, kRowMaxSlots] partial maxima of |SV| per frame and exit point
    int enc_slots[SMTM_MAX_EXITS];               // slots per frame the last encode of each exit point filled
    float* part;                                 // [tiles, 6, max_batch] per-tile best / second best of the last lookup
    bool sa_fresh;                               // no lookup yet in this batch: the next one overwrites SA
    bool begin_pending;                          // smtm_begin_batch has been called but its device work not enqueued yet:
                                                 // the first encode of the batch does it, or flush_begin() before anything else
    int32_t* live[2];                            // ping-pong live lists
    int cur;
    int32_t* next_slots;                         // old slot of each survivor
    int32_t* decision;
    int32_t* dlabel;
    float* top_val;
    int32_t* top_id;
    int32_t* res_layer;
    int32_t* res_label;
    int32_t* res_tier;
    Counts* counts;
    // update scratch
    uint32_t* cls_cnt;
    int32_t* cls_last;
    uint64_t* score;
    uint64_t* score_total;                       // [2] 128-bit sum of the scores
    int32_t* below;                              // [1] classes whose prefix share is below the confidence level
    int32_t* order;
    int32_t* all_exits;                          // [max_batch] filled with L: "stopped at the last exit point"
    // pinned staging for small host -> device copies: a ring of slots, each guarded by an event that is
    // recorded behind the copy that reads it, so that a call only waits when every slot is still in flight
    static constexpr int kStageSlots = 4;
    void* pinned;
    size_t pinned_bytes;                         // per slot
    hipEvent_t stage_ev[kStageSlots];
    bool stage_used[kStageSlots];
    int stage_next;

    // host-side bookkeeping
    int batch;                                   // 0 = no batch begun
    int stage_done[SMTM_MAX_EXITS];              // 0 none, 1 encoded, 2 looked up, 3 compacted
    int enc_dtype[SMTM_MAX_EXITS];
    char enc_kernel[SMTM_MAX_EXITS][96];         // name of the kernel instance the last encode of each exit point launched
    std::vector<void*> allocs;
};

static char g_create_err[512] = "";

static int32_t fail(smtm_ctx* ctx, int32_t code, const char* fmt, ...) {
    char* dst = ctx ? ctx->err : g_create_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(ctx, expr)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(ctx, e_ == hipErrorOutOfMemory ? SMTM_ERR_NOMEM : SMTM_ERR_HIP,      \
                        "%s failed: %s", #expr, hipGetErrorString(e_));                      \
    } while (0)

static int32_t check_launch(smtm_ctx* ctx, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ctx, SMTM_ERR_HIP, "%s: launch failed: %s", what, hipGetErrorString(e));
    return SMTM_OK;
}

template <typename T>
static hipError_t dev_alloc(smtm_ctx* ctx, T** p, size_t count) {
    void* q = nullptr;
    hipError_t e = hipMalloc(&q, count * sizeof(T) ? count * sizeof(T) : 1);
    if (e == hipSuccess) { ctx->allocs.push_back(q); *p = static_cast<T*>(q); }
    return e;
}

static int32_t validate_config(const smtm_config* c) {
    if (!c) return fail(nullptr, SMTM_ERR_INVALID_ARG, "config is NULL");
    if (c->n_classes < 2 || c->n_classes > SMTM_MAX_CLASSES)
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "n_classes %d outside 2..%d", c->n_classes, SMTM_MAX_CLASSES);
    if (c->n_exits < 1 || c->n_exits > SMTM_MAX_EXITS)
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "n_exits %d outside 1..%d", c->n_exits, SMTM_MAX_EXITS);
    for (int l = 0; l < c->n_exits; ++l)
        if (c->dims[l] < 1 || c->dims[l] > 65536)
            return fail(nullptr, SMTM_ERR_SHAPE, "dims[%d] = %d outside 1..65536", l, c->dims[l]);
    if (c->max_batch < 1 || c->max_batch > SMTM_MAX_BATCH)
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "max_batch %d outside 1..%d", c->max_batch, SMTM_MAX_BATCH);
    if (c->hot_min < 2 || c->hot_min > c->hot_init || c->hot_init > c->hot_max || c->hot_max > c->n_classes)
        return fail(nullptr, SMTM_ERR_INVALID_ARG,
                    "need 2 <= hot_min (%d) <= hot_init (%d) <= hot_max (%d) <= n_classes (%d)", c->hot_min,
                    c->hot_init, c->hot_max, c->n_classes);
    if (c->tiers != 1 && c->tiers != 2) return fail(nullptr, SMTM_ERR_INVALID_ARG, "tiers must be 1 or 2");
    if (!(c->tau >= 0.f) || !(c->tau < __builtin_inff()))
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "tau must be finite and >= 0");
    if (c->window < 1) return fail(nullptr, SMTM_ERR_INVALID_ARG, "window must be >= 1");
    if (c->cl_num < 1 || c->cl_den < c->cl_num)
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "need 0 < cl_num <= cl_den");
    if (c->init_count < 0) return fail(nullptr, SMTM_ERR_INVALID_ARG, "init_count must be >= 0");
    if (c->score_path < SMTM_SCORE_AUTO || c->score_path > SMTM_SCORE_MFMA)
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "score_path must be one of SMTM_SCORE_*");
    if (c->forgetting != SMTM_FORGET_AT_SCORING && c->forgetting != SMTM_FORGET_IN_PLACE)
        return fail(nullptr, SMTM_ERR_INVALID_ARG, "forgetting must be one of SMTM_FORGET_*");
    return SMTM_OK;
}

// Every call that touches the GPU starts here: the context's buffers live on one GPU, and a launch
// from a thread whose current device is another one would hand them to the wrong device.
static int32_t check_ctx(smtm_ctx* ctx) {
    if (!ctx) return fail(nullptr, SMTM_ERR_INVALID_ARG, "context is NULL");
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return fail(ctx, SMTM_ERR_STATE, "the context lives on GPU %d but the current device is %d", ctx->device, dev);
    return SMTM_OK;
}

static int32_t check_ctx_exit(smtm_ctx* ctx, int32_t exit) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (exit < 1 || exit > ctx->cfg.n_exits)
        return fail(ctx, SMTM_ERR_INVALID_ARG, "exit point %d outside 1..%d", exit, ctx->cfg.n_exits);
    return SMTM_OK;
}

extern "C" {

int32_t smtm_version(void) { return 200; }

#ifndef SMTM_BUILD_ID
#define SMTM_BUILD_ID "0000000000000000"
#endif
// The marker in front of the id lets the build script find it in the file without loading the library.
static const char kBuildId[] = "SMTM_BUILD_ID=" SMTM_BUILD_ID;
const char* smtm_build_id(void) { return kBuildId + 14; }

const char* smtm_encode_kernel(const smtm_ctx* ctx, int32_t exit) {
    if (!ctx || exit < 1 || exit > ctx->cfg.n_exits) return "";
    return ctx->enc_kernel[exit - 1];
}

const char* smtm_last_error(const smtm_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

int32_t smtm_create(smtm_ctx** out, const smtm_config* cfg) {
    if (!out) return fail(nullptr, SMTM_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int32_t rc = validate_config(cfg);
    if (rc != SMTM_OK) return rc;
    smtm_ctx* ctx = new (std::nothrow) smtm_ctx();
    if (!ctx) return fail(nullptr, SMTM_ERR_NOMEM, "host allocation failed");
    ctx->cfg = *cfg;
    ctx->err[0] = 0;
    const int n = cfg->n_classes, L = cfg->n_exits, B = cfg->max_batch;
    ctx->n_pad = round_up(n, kRowPad);
    ctx->tiles = (n + kScoreTileCols - 1) / kScoreTileCols;
    for (int l = 0; l < L; ++l) ctx->Cp[l] = round_up(cfg->dims[l], kKPad);
#define CREATE_TRY(expr)                                                                         \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) {                                                                  \
            rc = fail(nullptr, e_ == hipErrorOutOfMemory ? SMTM_ERR_NOMEM : SMTM_ERR_HIP,         \
                      "%s failed: %s", #expr, hipGetErrorString(e_));                            \
            smtm_destroy(ctx);                                                                   \
            return rc;                                                                           \
        }                                                                                        \
    } while (0)
    CREATE_TRY(hipGetDevice(&ctx->device));
    for (int l = 0; l < L; ++l) {
        const size_t C = cfg->dims[l];
        CREATE_TRY(dev_alloc(ctx, &ctx->centres[l], (size_t)n * C));
        CREATE_TRY(dev_alloc(ctx, &ctx->cinv[l], (size_t)n));
        CREATE_TRY(dev_alloc(ctx, &ctx->chat[l], (size_t)ctx->n_pad * ctx->Cp[l]));
        CREATE_TRY(dev_alloc(ctx, &ctx->mcount[l], (size_t)n));
        CREATE_TRY(dev_alloc(ctx, &ctx->sv[l], (size_t)B * ctx->Cp[l]));
        CREATE_TRY(dev_alloc(ctx, &ctx->slot_of[l], (size_t)B));
    }
    CREATE_TRY(dev_alloc(ctx, &ctx->FT, (size_t)n));
    CREATE_TRY(dev_alloc(ctx, &ctx->TS, (size_t)n));
    CREATE_TRY(dev_alloc(ctx, &ctx->hot_ids, (size_t)cfg->hot_max));
    CREATE_TRY(dev_alloc(ctx, &ctx->ids_stage, (size_t)cfg->hot_max));
    CREATE_TRY(dev_alloc(ctx, &ctx->in_hot, (size_t)ctx->n_pad));
    CREATE_TRY(dev_alloc(ctx, &ctx->SA, (size_t)B * n + kScoreTileCols));
    CREATE_TRY(dev_alloc(ctx, &ctx->rowmax, (size_t)L * B * kRowMaxSlots));
    CREATE_TRY(dev_alloc(ctx, &ctx->part, (size_t)ctx->tiles * 6 * B));
    CREATE_TRY(dev_alloc(ctx, &ctx->live[0], (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->live[1], (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->next_slots, (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->decision, (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->dlabel, (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->top_val, (size_t)B * 4));
    CREATE_TRY(dev_alloc(ctx, &ctx->top_id, (size_t)B * 2));
    CREATE_TRY(dev_alloc(ctx, &ctx->res_layer, (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->res_label, (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->res_tier, (size_t)B));
    CREATE_TRY(dev_alloc(ctx, &ctx->counts, (size_t)1));
    CREATE_TRY(dev_alloc(ctx, &ctx->cls_cnt, (size_t)n));
    CREATE_TRY(dev_alloc(ctx, &ctx->cls_last, (size_t)n));
    CREATE_TRY(dev_alloc(ctx, &ctx->score, (size_t)n));
    CREATE_TRY(dev_alloc(ctx, &ctx->order, (size_t)n));
    CREATE_TRY(dev_alloc(ctx, &ctx->score_total, (size_t)2));
    CREATE_TRY(dev_alloc(ctx, &ctx->below, (size_t)1));
    CREATE_TRY(dev_alloc(ctx, &ctx->all_exits, (size_t)B));
    ctx->pinned_bytes = sizeof(int32_t) * (size_t)cfg->hot_max;
    CREATE_TRY(hipHostMalloc(&ctx->pinned, ctx->pinned_bytes * smtm_ctx::kStageSlots, hipHostMallocDefault));
    for (int i = 0; i < smtm_ctx::kStageSlots; ++i) CREATE_TRY(hipEventCreateWithFlags(&ctx->stage_ev[i], hipEventDisableTiming));

    // initial state on the null stream: zero centres / tables, fast memory = classes 0..hot_init-1
    for (int l = 0; l < L; ++l) {
        CREATE_TRY(hipMemset(ctx->centres[l], 0, sizeof(float) * (size_t)n * cfg->dims[l]));
        CREATE_TRY(hipMemset(ctx->cinv[l], 0, sizeof(float) * (size_t)n));
        CREATE_TRY(hipMemset(ctx->chat[l], 0, sizeof(_Float16) * (size_t)ctx->n_pad * ctx->Cp[l]));
        CREATE_TRY(hipMemset(ctx->sv[l], 0, sizeof(float) * (size_t)B * ctx->Cp[l]));
        CREATE_TRY(hipMemset(ctx->slot_of[l], 0, sizeof(int32_t) * (size_t)B));
        launch_fill_u32(ctx->mcount[l], (uint32_t)cfg->init_count, n, nullptr);
    }
    launch_fill_u32(reinterpret_cast<uint32_t*>(ctx->all_exits), (uint32_t)L, B, nullptr);
    CREATE_TRY(hipMemset(ctx->FT, 0, sizeof(uint32_t) * (size_t)n));
    CREATE_TRY(hipMemset(ctx->TS, 0, sizeof(uint32_t) * (size_t)n));
    CREATE_TRY(hipMemset(ctx->counts, 0, sizeof(Counts)));
    CREATE_TRY(hipMemset(ctx->in_hot, 0, (size_t)ctx->n_pad));
    CREATE_TRY(hipMemset(ctx->rowmax, 0, sizeof(uint32_t) * (size_t)L * B * kRowMaxSlots));
    CREATE_TRY(hipMemset(ctx->part, 0, sizeof(float) * (size_t)ctx->tiles * 6 * B));
    CREATE_TRY(hipMemset(ctx->SA, 0, sizeof(float) * ((size_t)B * n + kScoreTileCols)));
    CREATE_TRY(hipMemset(ctx->live[0], 0, sizeof(int32_t) * (size_t)B));
    CREATE_TRY(hipMemset(ctx->live[1], 0, sizeof(int32_t) * (size_t)B));
    CREATE_TRY(hipMemset(ctx->next_slots, 0, sizeof(int32_t) * (size_t)B));
    CREATE_TRY(hipMemset(ctx->decision, 0, sizeof(int32_t) * (size_t)B));
    CREATE_TRY(hipMemset(ctx->dlabel, 0, sizeof(int32_t) * (size_t)B));
    {
        int32_t* ids = static_cast<int32_t*>(ctx->pinned);
        for (int i = 0; i < cfg->hot_init; ++i) ids[i] = i;
        CREATE_TRY(hipMemcpy(ctx->ids_stage, ids, sizeof(int32_t) * (size_t)cfg->hot_init, hipMemcpyHostToDevice));
        launch_set_hot(ctx->ids_stage, cfg->hot_init, n, ctx->hot_ids, ctx->in_hot, ctx->counts, nullptr);
    }
    CREATE_TRY(hipGetLastError());
    CREATE_TRY(hipDeviceSynchronize());
#undef CREATE_TRY
    ctx->batch = 0;
    ctx->cur = 0;
    *out = ctx;
    return SMTM_OK;
}

int32_t smtm_destroy(smtm_ctx* ctx) {
    if (!ctx) return SMTM_OK;
    (void)hipDeviceSynchronize();
    for (void* p : ctx->allocs) (void)hipFree(p);
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    for (int i = 0; i < smtm_ctx::kStageSlots; ++i)
        if (ctx->stage_ev[i]) (void)hipEventDestroy(ctx->stage_ev[i]);
    delete ctx;
    return SMTM_OK;
}

int32_t smtm_memory_load(smtm_ctx* ctx, int32_t exit, const float* centres_host, void* stream) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    if (!centres_host) return fail(ctx, SMTM_ERR_INVALID_ARG, "centres_host is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int l = exit - 1, n = ctx->cfg.n_classes, C = ctx->cfg.dims[l];
    HIP_TRY(ctx, hipMemcpyAsync(ctx->centres[l], centres_host, sizeof(float) * (size_t)n * C, hipMemcpyHostToDevice, st));
    launch_centre_prepare(ctx->centres[l], n, C, ctx->cinv[l], ctx->chat[l], ctx->Cp[l], 0, ctx->n_pad, st);
    launch_fill_u32(ctx->mcount[l], (uint32_t)ctx->cfg.init_count, n, st);
    return check_launch(ctx, "smtm_memory_load");
}

int32_t smtm_memory_import(smtm_ctx* ctx, int32_t exit, const float* centres_host, const uint32_t* counts_host,
                           void* stream) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    if (!centres_host || !counts_host) return fail(ctx, SMTM_ERR_INVALID_ARG, "centres_host / counts_host is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int l = exit - 1, n = ctx->cfg.n_classes, C = ctx->cfg.dims[l];
    HIP_TRY(ctx, hipMemcpyAsync(ctx->centres[l], centres_host, sizeof(float) * (size_t)n * C, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(ctx->mcount[l], counts_host, sizeof(uint32_t) * (size_t)n, hipMemcpyHostToDevice, st));
    launch_centre_prepare(ctx->centres[l], n, C, ctx->cinv[l], ctx->chat[l], ctx->Cp[l], 0, ctx->n_pad, st);
    return check_launch(ctx, "smtm_memory_import");
}

int32_t smtm_hot_set(smtm_ctx* ctx, const int32_t* ids, int32_t k, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (!ids) return fail(ctx, SMTM_ERR_INVALID_ARG, "class_ids_host is NULL");
    if (k < ctx->cfg.hot_min || k > ctx->cfg.hot_max)
        return fail(ctx, SMTM_ERR_INVALID_ARG, "k = %d outside hot_min..hot_max (%d..%d)", k, ctx->cfg.hot_min, ctx->cfg.hot_max);
    std::vector<uint8_t> seen((size_t)ctx->cfg.n_classes, 0);
    for (int i = 0; i < k; ++i) {
        if (ids[i] < 0 || ids[i] >= ctx->cfg.n_classes) return fail(ctx, SMTM_ERR_INVALID_ARG, "class id %d out of range", ids[i]);
        if (seen[ids[i]]) return fail(ctx, SMTM_ERR_INVALID_ARG, "class id %d listed twice", ids[i]);
        seen[ids[i]] = 1;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    // next staging slot; the host waits only if the copy that last read this slot has not run yet
    const int slot = ctx->stage_next;
    ctx->stage_next = (slot + 1) % smtm_ctx::kStageSlots;
    if (ctx->stage_used[slot]) HIP_TRY(ctx, hipEventSynchronize(ctx->stage_ev[slot]));
    void* stage = static_cast<char*>(ctx->pinned) + ctx->pinned_bytes * (size_t)slot;
    memcpy(stage, ids, sizeof(int32_t) * (size_t)k);
    HIP_TRY(ctx, hipMemcpyAsync(ctx->ids_stage, stage, sizeof(int32_t) * (size_t)k, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipEventRecord(ctx->stage_ev[slot], st));
    ctx->stage_used[slot] = true;
    launch_set_hot(ctx->ids_stage, k, ctx->cfg.n_classes, ctx->hot_ids, ctx->in_hot, ctx->counts, st);
    return check_launch(ctx, "smtm_hot_set");
}

int32_t smtm_memory_export(smtm_ctx* ctx, int32_t exit, float* centres_host, uint32_t* counts_host, void* stream) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int l = exit - 1, n = ctx->cfg.n_classes, C = ctx->cfg.dims[l];
    if (centres_host) HIP_TRY(ctx, hipMemcpyAsync(centres_host, ctx->centres[l], sizeof(float) * (size_t)n * C, hipMemcpyDeviceToHost, st));
    if (counts_host) HIP_TRY(ctx, hipMemcpyAsync(counts_host, ctx->mcount[l], sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    return SMTM_OK;
}

int32_t smtm_tables_export(smtm_ctx* ctx, uint32_t* ft, uint32_t* ts, int32_t* hot_ids, int32_t* k, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n = ctx->cfg.n_classes;
    Counts c;
    if (ft) HIP_TRY(ctx, hipMemcpyAsync(ft, ctx->FT, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
    if (ts) HIP_TRY(ctx, hipMemcpyAsync(ts, ctx->TS, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
    if (hot_ids) HIP_TRY(ctx, hipMemcpyAsync(hot_ids, ctx->hot_ids, sizeof(int32_t) * (size_t)ctx->cfg.hot_max, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(&c, ctx->counts, sizeof(Counts), hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    if (k) *k = c.hot_k;
    return SMTM_OK;
}

int32_t smtm_tables_import(smtm_ctx* ctx, const uint32_t* ft, const uint32_t* ts, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n = ctx->cfg.n_classes;
    if (ft) HIP_TRY(ctx, hipMemcpyAsync(ctx->FT, ft, sizeof(uint32_t) * (size_t)n, hipMemcpyHostToDevice, st));
    if (ts) HIP_TRY(ctx, hipMemcpyAsync(ctx->TS, ts, sizeof(uint32_t) * (size_t)n, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    return SMTM_OK;
}

int32_t smtm_set_tau(smtm_ctx* ctx, float tau) {
    if (!ctx) return fail(nullptr, SMTM_ERR_INVALID_ARG, "context is NULL");
    if (!(tau >= 0.f) || !(tau < __builtin_inff())) return fail(ctx, SMTM_ERR_INVALID_ARG, "tau must be finite and >= 0");
    ctx->cfg.tau = tau;
    return SMTM_OK;
}

int32_t smtm_begin_batch(smtm_ctx* ctx, int32_t batch, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (batch < 1 || batch > ctx->cfg.max_batch)
        return fail(ctx, SMTM_ERR_SHAPE, "batch %d outside 1..max_batch (%d)", batch, ctx->cfg.max_batch);
    (void)stream;                                // nothing is enqueued here, see begin_pending
    ctx->cur = 0;
    ctx->begin_pending = true;
    ctx->batch = batch;
    ctx->sa_fresh = true;
    for (int l = 0; l < SMTM_MAX_EXITS; ++l) ctx->stage_done[l] = 0;
    return SMTM_OK;
}

// The device side of smtm_begin_batch, for calls that are not an encode (an encode folds it into its kernel).
static void flush_begin(smtm_ctx* ctx, hipStream_t st) {
    if (!ctx->begin_pending) return;
    launch_begin_batch(ctx->batch, ctx->live[0], ctx->res_layer, ctx->res_label, ctx->res_tier, ctx->counts, st);
    ctx->begin_pending = false;
}

static int32_t check_encode_args(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    if (ctx->batch == 0) return fail(ctx, SMTM_ERR_STATE, "smtm_begin_batch has not been called");
    if (!fmap) return fail(ctx, SMTM_ERR_INVALID_ARG, "fmap is NULL");
    if ((reinterpret_cast<uintptr_t>(fmap) & 15u) != 0) return fail(ctx, SMTM_ERR_INVALID_ARG, "fmap must be 16-byte aligned");
    if (dtype != SMTM_F16 && dtype != SMTM_F32) return fail(ctx, SMTM_ERR_UNSUPPORTED, "dtype %d is neither SMTM_F16 nor SMTM_F32", dtype);
    if (H < 1 || W < 1 || (int64_t)H * W > (1 << 24)) return fail(ctx, SMTM_ERR_SHAPE, "H x W = %d x %d not supported", H, W);
    return SMTM_OK;
}

static int32_t encode_any(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W,
                          const int32_t* row_ids, float* sv_out, void* stream, bool channels_last) {
    int32_t rc = check_encode_args(ctx, exit, fmap, dtype, H, W);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int l = exit - 1;
    uint32_t* rowmax = ctx->rowmax + (size_t)l * ctx->cfg.max_batch * kRowMaxSlots;
    EncodeOut out = {};
    out.sv = ctx->sv[l]; out.ldv = ctx->Cp[l]; out.slot_of = ctx->slot_of[l]; out.sv_out = sv_out; out.rowmax = rowmax;
    if (ctx->begin_pending) {
        out.fresh = ctx->batch; out.live0 = ctx->live[0];
        out.res_layer = ctx->res_layer; out.res_label = ctx->res_label; out.res_tier = ctx->res_tier;
        out.counts_w = ctx->counts;
        // the context's own list as row ids would be read before this kernel has written it: it is the identity
        if (row_ids == ctx->live[0]) row_ids = nullptr;
    }
    if (channels_last)
        launch_encode_nhwc(fmap, dtype, ctx->cfg.dims[l], H * W, row_ids, ctx->live[ctx->cur], ctx->counts,
                           ctx->batch, out, st, ctx->enc_kernel[l], sizeof(ctx->enc_kernel[l]), &ctx->enc_slots[l]);
    else
        launch_encode(fmap, dtype, ctx->cfg.dims[l], H * W, row_ids, ctx->live[ctx->cur], ctx->counts, ctx->batch,
                      out, st, ctx->enc_kernel[l], sizeof(ctx->enc_kernel[l]), &ctx->enc_slots[l]);
    rc = check_launch(ctx, "smtm_encode");
    if (rc) return rc;
    ctx->begin_pending = false;
    ctx->stage_done[l] = 1;
    ctx->enc_dtype[l] = dtype;
    return SMTM_OK;
}

// --- lookup and exit/compact share these helpers ------------------------------------------

static int32_t check_lookup_state(smtm_ctx* ctx, int32_t exit, const char* who) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    if (ctx->batch == 0 || ctx->stage_done[exit - 1] != 1)
        return fail(ctx, SMTM_ERR_STATE, "%s(%d) needs smtm_encode(%d) first, once per batch", who, exit, exit);
    return SMTM_OK;
}

static int32_t check_compact_args(smtm_ctx* ctx, const int32_t* live_ids, const void* fmap_in,
                                  const int32_t* row_ids, const void* fmap_out, int64_t row_bytes) {
    if ((fmap_in != nullptr) != (fmap_out != nullptr))
        return fail(ctx, SMTM_ERR_INVALID_ARG, "fmap_in and fmap_out must be given together");
    if (fmap_out) {
        if (row_bytes < 2 || (row_bytes & 1)) return fail(ctx, SMTM_ERR_SHAPE, "row_bytes %lld must be even and >= 2", (long long)row_bytes);
        if (((reinterpret_cast<uintptr_t>(fmap_in) | reinterpret_cast<uintptr_t>(fmap_out)) & 15u) != 0)
            return fail(ctx, SMTM_ERR_INVALID_ARG, "fmap_in and fmap_out must be 16-byte aligned");
        if (fmap_in == fmap_out) return fail(ctx, SMTM_ERR_INVALID_ARG, "fmap_out must not overlap fmap_in");
    }
    const int32_t* cur = ctx->live[ctx->cur];
    const int32_t* nxt = ctx->live[ctx->cur ^ 1];
    if (live_ids == cur || live_ids == nxt || row_ids == nxt)
        return fail(ctx, SMTM_ERR_INVALID_ARG, "live_ids / row_ids alias the context's next live list");
    return SMTM_OK;
}

constexpr int kFusedDecideRows = 2048;   // largest batch whose decisions are made inside the compaction kernel

static CompactArgs compact_args(smtm_ctx* ctx, int32_t exit, int32_t* exit_ids, int32_t* exit_labels,
                                int32_t* exit_tier, int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev) {
    CompactArgs a;
    a.decision = ctx->decision; a.label = ctx->dlabel; a.frame_ids = ctx->live[ctx->cur];
    a.next_ids = ctx->live[ctx->cur ^ 1]; a.next_slots = ctx->next_slots; a.counts = ctx->counts;
    a.max_rows = ctx->batch;
    a.exit_index = exit;
    a.exit_ids = exit_ids; a.exit_labels = exit_labels; a.exit_tier = exit_tier; a.n_exit_dev = n_exit_dev;
    a.live_ids_user = live_ids; a.n_live_dev = n_live_dev;
    a.res_layer = ctx->res_layer; a.res_label = ctx->res_label; a.res_tier = ctx->res_tier;
    return a;
}

// scores, SA accumulation and the per-tile best / second best (one launch)
static void enqueue_score(smtm_ctx* ctx, int32_t exit, float* sims_out, hipStream_t st) {
    const int l = exit - 1;
    int path = ctx->cfg.score_path;
    if (path == SMTM_SCORE_AUTO) path = ctx->enc_dtype[l] == SMTM_F16 ? SMTM_SCORE_MFMA : SMTM_SCORE_FP32;
    ScoreArgs a;
    a.sv = ctx->sv[l]; a.ldv = ctx->Cp[l];
    a.rowmax = ctx->rowmax + (size_t)l * ctx->cfg.max_batch * kRowMaxSlots;
    a.rowmax_slots = ctx->enc_slots[l];
    a.frame_ids = ctx->live[ctx->cur]; a.counts = ctx->counts; a.max_rows = ctx->batch;
    a.n = ctx->cfg.n_classes; a.weight = ldexpf(1.0f, exit - 1);
    a.first = ctx->sa_fresh ? 1 : 0;
    a.SA = ctx->SA; a.sims_out = sims_out; a.in_hot = ctx->in_hot;
    a.part = ctx->part; a.part_stride = ctx->cfg.max_batch;
    if (path == SMTM_SCORE_MFMA) launch_score_mfma(a, ctx->chat[l], ctx->Cp[l], st);
    else launch_score_fp32(a, ctx->centres[l], ctx->cinv[l], ctx->cfg.dims[l], st);
    ctx->sa_fresh = false;
}

static DecideArgs decide_args(smtm_ctx* ctx, float* top_val, int32_t* top_id) {
    DecideArgs g;
    g.part = ctx->part; g.part_stride = ctx->cfg.max_batch; g.tiles = ctx->tiles;
    g.counts = ctx->counts; g.max_rows = ctx->batch; g.tiers = ctx->cfg.tiers; g.tau = ctx->cfg.tau;
    g.decision = ctx->decision; g.label = ctx->dlabel; g.top_val = ctx->top_val; g.top_id = ctx->top_id;
    g.top_val_user = top_val; g.top_id_user = top_id;
    return g;
}

int32_t smtm_lookup(smtm_ctx* ctx, int32_t exit, float* top_val, int32_t* top_id, float* sims_out, void* stream) {
    int32_t rc = check_lookup_state(ctx, exit, "smtm_lookup");
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    enqueue_score(ctx, exit, sims_out, st);
    launch_decide(decide_args(ctx, top_val, top_id), st);
    rc = check_launch(ctx, "smtm_lookup");
    if (rc) return rc;
    ctx->stage_done[exit - 1] = 2;
    return SMTM_OK;
}

int32_t smtm_separability(smtm_ctx* ctx, int32_t exit, const float* sims, float* sep_out, void* stream) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    if (!sims || !sep_out) return fail(ctx, SMTM_ERR_INVALID_ARG, "sims / sep_out is NULL");
    if (ctx->batch == 0 || ctx->stage_done[exit - 1] != 2)
        return fail(ctx, SMTM_ERR_STATE, "smtm_separability(%d) goes between smtm_lookup(%d) and smtm_exit_compact(%d)", exit, exit, exit);
    launch_separability(sims, ctx->counts, ctx->batch, ctx->cfg.n_classes, ctx->in_hot, sep_out,
                        static_cast<hipStream_t>(stream));
    return check_launch(ctx, "smtm_separability");
}

int32_t smtm_exit_compact(smtm_ctx* ctx, int32_t exit, int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                          int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev, const void* fmap_in,
                          const int32_t* row_ids, void* fmap_out, int64_t row_bytes, void* stream) {
    int32_t rc = check_ctx_exit(ctx, exit);
    if (rc) return rc;
    const int l = exit - 1;
    if (ctx->batch == 0 || ctx->stage_done[l] != 2)
        return fail(ctx, SMTM_ERR_STATE, "smtm_exit_compact(%d) needs smtm_lookup(%d) first, once per batch", exit, exit);
    rc = check_compact_args(ctx, live_ids, fmap_in, row_ids, fmap_out, row_bytes);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    launch_compact(compact_args(ctx, exit, exit_ids, exit_labels, exit_tier, n_exit_dev, live_ids, n_live_dev), st);
    if (fmap_out)
        launch_gather_rows(fmap_in, row_ids, ctx->next_slots, ctx->counts, ctx->batch, fmap_out, row_bytes, st);
    rc = check_launch(ctx, "smtm_exit_compact");
    if (rc) return rc;
    ctx->cur ^= 1;
    ctx->stage_done[l] = 3;
    return SMTM_OK;
}

int32_t smtm_lookup_exit(smtm_ctx* ctx, int32_t exit, float* top_val, int32_t* top_id,
                         int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier, int32_t* n_exit_dev,
                         int32_t* live_ids, int32_t* n_live_dev, const void* fmap_in, const int32_t* row_ids,
                         void* fmap_out, int64_t row_bytes, void* stream) {
    int32_t rc = check_lookup_state(ctx, exit, "smtm_lookup_exit");
    if (rc) return rc;
    rc = check_compact_args(ctx, live_ids, fmap_in, row_ids, fmap_out, row_bytes);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    enqueue_score(ctx, exit, nullptr, st);
    // The fused kernel is one block: it merges a slot's per-tile results on one CU, which for a long batch takes
    // longer than a launch (14 against 12 us at 4096 frames).  Long batches decide on many CUs first.
    if (ctx->batch > kFusedDecideRows) {
        launch_decide(decide_args(ctx, top_val, top_id), st);
        launch_compact(compact_args(ctx, exit, exit_ids, exit_labels, exit_tier, n_exit_dev, live_ids, n_live_dev), st);
    } else {
        launch_decide_compact(decide_args(ctx, top_val, top_id),
                              compact_args(ctx, exit, exit_ids, exit_labels, exit_tier, n_exit_dev, live_ids, n_live_dev), st);
    }
    if (fmap_out)
        launch_gather_rows(fmap_in, row_ids, ctx->next_slots, ctx->counts, ctx->batch, fmap_out, row_bytes, st);
    rc = check_launch(ctx, "smtm_lookup_exit");
    if (rc) return rc;
    ctx->cur ^= 1;
    ctx->stage_done[exit - 1] = 3;
    return SMTM_OK;
}

static int32_t stage_any(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W,
                         const int32_t* row_ids, int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                         int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev, void* fmap_out, void* stream,
                         bool channels_last) {
    int32_t rc = check_encode_args(ctx, exit, fmap, dtype, H, W);
    if (rc) return rc;
    const int l = exit - 1;
    const int64_t row_bytes = (int64_t)ctx->cfg.dims[l] * H * W * (dtype == SMTM_F16 ? 2 : 4);
    rc = check_compact_args(ctx, live_ids, fmap_out ? fmap : nullptr, row_ids, fmap_out, row_bytes);
    if (rc) return rc;
    rc = encode_any(ctx, exit, fmap, dtype, H, W, row_ids, nullptr, stream, channels_last);
    if (rc) return rc;
    return smtm_lookup_exit(ctx, exit, nullptr, nullptr, exit_ids, exit_labels, exit_tier, n_exit_dev, live_ids,
                            n_live_dev, fmap_out ? fmap : nullptr, row_ids, fmap_out, row_bytes, stream);
}

int32_t smtm_stage(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W,
                   const int32_t* row_ids, int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                   int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev, void* fmap_out, void* stream) {
    return stage_any(ctx, exit, fmap, dtype, H, W, row_ids, exit_ids, exit_labels, exit_tier, n_exit_dev, live_ids,
                     n_live_dev, fmap_out, stream, false);
}

int32_t smtm_stage_nhwc(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W,
                        const int32_t* row_ids, int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                        int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev, void* fmap_out, void* stream) {
    return stage_any(ctx, exit, fmap, dtype, H, W, row_ids, exit_ids, exit_labels, exit_tier, n_exit_dev, live_ids,
                     n_live_dev, fmap_out, stream, true);
}

int32_t smtm_encode(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W,
                    const int32_t* row_ids, float* sv_out, void* stream) {
    return encode_any(ctx, exit, fmap, dtype, H, W, row_ids, sv_out, stream, false);
}

int32_t smtm_encode_nhwc(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype, int32_t H, int32_t W,
                         const int32_t* row_ids, float* sv_out, void* stream) {
    return encode_any(ctx, exit, fmap, dtype, H, W, row_ids, sv_out, stream, true);
}

const int32_t* smtm_live_ids(const smtm_ctx* ctx) { return ctx ? ctx->live[ctx->cur] : nullptr; }

int32_t smtm_batch_results(smtm_ctx* ctx, int32_t* exit_layer, int32_t* label, int32_t* tier, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (ctx->batch == 0) return fail(ctx, SMTM_ERR_STATE, "smtm_begin_batch has not been called");
    hipStream_t st = static_cast<hipStream_t>(stream);
    flush_begin(ctx, st);
    launch_copy3_i32(ctx->res_layer, exit_layer, ctx->res_label, label, ctx->res_tier, tier, ctx->batch, st);
    return check_launch(ctx, "smtm_batch_results");
}

int32_t smtm_read_counts(smtm_ctx* ctx, int32_t* n_live_host, int32_t* n_exit_host, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    flush_begin(ctx, st);
    Counts c;
    HIP_TRY(ctx, hipMemcpyAsync(&c, ctx->counts, sizeof(Counts), hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    if (n_live_host) *n_live_host = c.n_live;
    if (n_exit_host) *n_exit_host = c.n_exit;
    return SMTM_OK;
}

int32_t smtm_read_stats(smtm_ctx* ctx, int32_t* stats_host, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (!stats_host) return fail(ctx, SMTM_ERR_INVALID_ARG, "stats_host is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    flush_begin(ctx, st);
    Counts c;
    HIP_TRY(ctx, hipMemcpyAsync(&c, ctx->counts, sizeof(Counts), hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    for (int l = 0; l < ctx->cfg.n_exits; ++l)
        for (int i = 0; i < 4; ++i) stats_host[l * 4 + i] = c.stats[l][i];
    return SMTM_OK;
}

static CentreTables centre_tables(const smtm_ctx* ctx) {
    CentreTables tabs;
    for (int l = 0; l < SMTM_MAX_EXITS; ++l) {
        const bool on = l < ctx->cfg.n_exits;
        tabs.centres[l] = on ? ctx->centres[l] : nullptr;
        tabs.mcount[l] = on ? ctx->mcount[l] : nullptr;
        tabs.cinv[l] = on ? ctx->cinv[l] : nullptr;
        tabs.chat[l] = on ? ctx->chat[l] : nullptr;
        tabs.sv[l] = on ? ctx->sv[l] : nullptr;
        tabs.slot_of[l] = on ? ctx->slot_of[l] : nullptr;
        tabs.C[l] = on ? ctx->cfg.dims[l] : 0;
        tabs.Cp[l] = on ? ctx->Cp[l] : 0;
    }
    tabs.res_layer = ctx->res_layer;
    int upto = 0;
    while (upto < ctx->cfg.n_exits && ctx->stage_done[upto] >= 1) ++upto;
    tabs.enc_upto = upto;
    return tabs;
}

int32_t smtm_warmup_begin(smtm_ctx* ctx, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n = ctx->cfg.n_classes;
    for (int l = 0; l < ctx->cfg.n_exits; ++l) {
        launch_fill_u32(reinterpret_cast<uint32_t*>(ctx->centres[l]), 0u, n * ctx->cfg.dims[l], st);
        launch_fill_u32(ctx->mcount[l], 0u, n, st);
        launch_centre_prepare(ctx->centres[l], n, ctx->cfg.dims[l], ctx->cinv[l], ctx->chat[l], ctx->Cp[l], 0, ctx->n_pad, st);
    }
    return check_launch(ctx, "smtm_warmup_begin");
}

int32_t smtm_warmup_batch(smtm_ctx* ctx, const int32_t* label, int32_t batch, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (!label) return fail(ctx, SMTM_ERR_INVALID_ARG, "label is NULL");
    if (ctx->batch == 0) return fail(ctx, SMTM_ERR_STATE, "smtm_begin_batch has not been called");
    if (batch != ctx->batch) return fail(ctx, SMTM_ERR_SHAPE, "batch %d differs from the batch begun (%d)", batch, ctx->batch);
    for (int l = 0; l < ctx->cfg.n_exits; ++l)
        if (ctx->stage_done[l] != 1)
            return fail(ctx, SMTM_ERR_STATE, "smtm_warmup_batch needs smtm_encode (and nothing else) at every exit point of this batch; exit point %d is missing", l + 1);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n = ctx->cfg.n_classes;
    launch_class_count(label, batch, n, ctx->cls_cnt, st);
    launch_centres_update(centre_tables(ctx), ctx->cfg.n_exits, n, label, ctx->all_exits, batch, ctx->cls_cnt, st);
    int32_t rc = check_launch(ctx, "smtm_warmup_batch");
    if (rc) return rc;
    for (int l = 0; l < ctx->cfg.n_exits; ++l) ctx->stage_done[l] = 3;     // the batch has been used
    return SMTM_OK;
}

static int32_t cache_update_with(smtm_ctx* ctx, const int32_t* label, const int32_t* stop_layer, int32_t batch,
                                 void* stream, const UpdateScratch& us, const char* who) {
    if ((label == nullptr) != (stop_layer == nullptr))
        return fail(ctx, SMTM_ERR_INVALID_ARG, "label and stop_layer must be given together (or both NULL)");
    if (ctx->batch == 0) return fail(ctx, SMTM_ERR_STATE, "smtm_begin_batch has not been called");
    if (!label) { label = ctx->res_label; stop_layer = ctx->res_layer; }     // the batch's own exits
    if (batch != ctx->batch) return fail(ctx, SMTM_ERR_SHAPE, "batch %d differs from the batch begun (%d)", batch, ctx->batch);
    hipStream_t st = static_cast<hipStream_t>(stream);
    flush_begin(ctx, st);
    const smtm_config& c = ctx->cfg;
    const int n = c.n_classes;
    launch_tables_update(label, batch, n, (uint32_t)c.window, ctx->FT, ctx->TS, us.cls_cnt, us.cls_last,
                         us.score, us.total, us.below, c.forgetting, st);
    launch_centres_and_policy(centre_tables(ctx), c.n_exits, n, label, stop_layer, batch, us.cls_cnt, us.score,
                              us.total, (uint32_t)c.cl_num, (uint32_t)c.cl_den, c.hot_min, c.hot_max,
                              us.order, us.below, ctx->hot_ids, ctx->in_hot, ctx->counts, st);
    return check_launch(ctx, who);
}

int32_t smtm_cache_update(smtm_ctx* ctx, const int32_t* label, const int32_t* stop_layer, int32_t batch, void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    const UpdateScratch us = {ctx->cls_cnt, ctx->cls_last, ctx->score, ctx->order, ctx->score_total, ctx->below};
    return cache_update_with(ctx, label, stop_layer, batch, stream, us, "smtm_cache_update");
}

int32_t smtm_cache_update_static(smtm_ctx* ctx, const int32_t* label, const int32_t* stop_layer, int32_t batch,
                                 void* stream) {
    if (int32_t rc = check_ctx(ctx)) return rc;
    if (ctx->cfg.n_classes > kStaticMaxClasses)
        return fail(ctx, SMTM_ERR_UNSUPPORTED, "smtm_cache_update_static holds scratch for at most %d classes, the context has %d",
                    kStaticMaxClasses, ctx->cfg.n_classes);
    UpdateScratch us;
    const hipError_t e = update_static_scratch(ctx->device, &us);
    if (e != hipSuccess) return fail(ctx, SMTM_ERR_HIP, "address of the static scratch: %s", hipGetErrorString(e));
    return cache_update_with(ctx, label, stop_layer, batch, stream, us, "smtm_cache_update_static");
}

}  // extern "C"
