/*
 * smtm.h — C ABI of the MI355X (gfx950) library for the batched hot path of semantic-memory
 * CNN inference (arXiv 2112.02644, "SMTM"): at every exit point a batch of frames is
 *   1. encoded: each feature map is pooled to a semantic vector        (Sec. 4.1)
 *   2. looked up: cosine similarity against every class centre (Eq. 1), accumulated over
 *      exit points with weights 2^(l-1) (Eq. 3), best and second best per memory tier
 *   3. released or kept: accumulated confidence against the threshold (Eq. 4); frames that
 *      exit are listed, the others are compacted so they continue through the network
 * and between batches the memory is updated: frequency / time-stamp tables and the
 * replacement score (Sec. 6.1, Eq. 5), adaptive fast-memory size (Eq. 6), adaptive
 * centres (Eq. 7).
 *
 * Conventions
 *   - Plain C.  Every call returns an int32_t status (SMTM_OK or an SMTM_ERR_* code);
 *     smtm_last_error() gives a text for the last failure on that context.
 *   - Arguments are validated before any GPU work is enqueued; a failed call enqueues nothing.
 *   - "device" pointers are GPU memory owned by the caller (never freed or kept by the
 *     library beyond the stream-ordered completion of the call); "host" pointers are ordinary
 *     memory.  The context owns the memory tables, the accumulated similarities, the saved
 *     semantic vectors, the live list and the counters.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Hot calls only
 *     enqueue; they never synchronise.  All calls on one context must be issued on one stream
 *     (or be otherwise ordered by the caller).  A context is bound to the GPU that was current
 *     when it was created; calls made while another GPU is current fail with SMTM_ERR_STATE.
 *   - Exit points are numbered 1..L in network order; that number is the l of weight 2^(l-1).
 *     Classes are 0..n-1.  Frames of a batch are 0..batch-1 ("original frame id").
 *     "Slot" i is the i-th live frame, live frames being kept in ascending original id.
 */
#ifndef SMTM_H
#define SMTM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SMTM_OK               0
#define SMTM_ERR_INVALID_ARG  1   /* null pointer, value out of range */
#define SMTM_ERR_SHAPE        2   /* sizes that do not fit the context or each other */
#define SMTM_ERR_STATE        3   /* call order (e.g. lookup before encode of that exit point) */
#define SMTM_ERR_UNSUPPORTED  4
#define SMTM_ERR_NOMEM        5
#define SMTM_ERR_HIP          6   /* a HIP runtime call failed; text in smtm_last_error */

#define SMTM_F16 0
#define SMTM_F32 1

#define SMTM_MAX_EXITS    8
#define SMTM_MAX_CLASSES  16384
#define SMTM_MAX_BATCH    65536

/* how the similarities of Eq. 1 are computed */
#define SMTM_SCORE_AUTO   0   /* fp16 feature maps -> MFMA, fp32 feature maps -> FP32 */
#define SMTM_SCORE_FP32   1   /* fp32 operands, fp32 vector arithmetic */
#define SMTM_SCORE_MFMA   2   /* fp16 operands on the matrix cores (unit centres; semantic vectors scaled by a
                                 power of two, their length taken in fp32), fp32 accumulate */

/* how the forgetting of Sec. 6.1 acts on the frequency table */
#define SMTM_FORGET_AT_SCORING 0   /* Eq. 5: Score = FT * 0.25^floor(TS/W), FT itself keeps the whole history */
#define SMTM_FORGET_IN_PLACE   1   /* Sec. 6.1 text / Sec. 8.1: every W-th consecutive frame without class i
                                      replaces FT_i by floor(FT_i / 4); Score = FT */

typedef struct smtm_ctx smtm_ctx;

typedef struct {
    int32_t n_classes;               /* n: size of the global memory, 2..SMTM_MAX_CLASSES */
    int32_t n_exits;                 /* L: 1..SMTM_MAX_EXITS */
    int32_t dims[SMTM_MAX_EXITS];    /* C_l: channels (= semantic-vector length) at exit point l */
    int32_t max_batch;               /* largest batch, 1..SMTM_MAX_BATCH */
    int32_t hot_init;                /* initial size k of the fast memory; classes 0..k-1 until smtm_hot_set */
    int32_t hot_min, hot_max;        /* bounds of the adaptive size, 2 <= hot_min <= hot_init <= hot_max <= n */
    int32_t tiers;                   /* 1: fast memory only (Sec. 6); 2: fast memory, then global memory */
    float   tau;                     /* threshold of Eq. 4, >= 0 */
    int32_t window;                  /* W of Eq. 5 in frames, >= 1 */
    int32_t cl_num, cl_den;          /* confidence level of Eq. 6 as a fraction, 0 < cl_num <= cl_den (19/20) */
    int32_t init_count;              /* update count m every centre starts with (Eq. 7), >= 0 */
    int32_t score_path;              /* SMTM_SCORE_* */
    int32_t forgetting;              /* SMTM_FORGET_* */
} smtm_config;

/* ---- life cycle ------------------------------------------------------------------------- */

/* Allocates a context and its device memory on the current GPU.  *out is NULL on failure.
 * Errors: INVALID_ARG / SHAPE for a bad config (checked first, no GPU needed), HIP, NOMEM. */
int32_t smtm_create(smtm_ctx** out, const smtm_config* cfg);
/* Frees everything; synchronises the device first.  NULL is allowed. */
int32_t smtm_destroy(smtm_ctx* ctx);
/* Text of the last error on ctx (or of the last failed smtm_create when ctx is NULL).
 * The pointer stays valid until the next failing call. */
const char* smtm_last_error(const smtm_ctx* ctx);
/* Library version, major*10000 + minor*100 + patch. */
int32_t smtm_version(void);
/* Hash (16 hex digits) of the sources the library was built from; the Python binding compares it with
 * the sources in the tree and rebuilds a stale library. */
const char* smtm_build_id(void);

/* ---- memory (Sec. 6: global memory, fast memory) ----------------------------------------- */

/* Loads the semantic centres SC_j^l of exit point `exit`: host, [n, C_l] fp32 row-major,
 * copied (the host buffer must stay valid until the stream has passed this call).  Centres
 * need not be unit length.  Resets that exit point's update counts to init_count. */
int32_t smtm_memory_load(smtm_ctx* ctx, int32_t exit, const float* centres_host, void* stream);
/* Warm-up (Sec. 5, Sec. 6.3): centres initialised as the average of the semantic vectors of labelled
 * training frames, update counts as the number of samples per class.
 *   smtm_warmup_begin  sets every centre to 0 and every update count to 0.
 *   smtm_warmup_batch  adds one labelled batch: call smtm_begin_batch, then smtm_encode at every exit
 *                      point (all frames live, no lookup), then this with label[b] (device int32
 *                      [batch], class of frame b or -1 to skip it).  Centres move to the running mean
 *                      (SC*m + sum of SV)/(m + count), which after the last batch is the class mean.
 * Classes that never appear keep the zero vector (similarity 0 to everything).  Nothing else of the
 * memory (tables, fast-memory set) is touched.  Errors: STATE when an exit point of the batch has not
 * been encoded (or has been looked up), SHAPE when batch differs from the batch begun. */
int32_t smtm_warmup_begin(smtm_ctx* ctx, void* stream);
int32_t smtm_warmup_batch(smtm_ctx* ctx, const int32_t* label, int32_t batch, void* stream);
/* Restores one exit point's centres AND their update counts m (Eq. 7) from host buffers, as written by
 * smtm_memory_export: [n, C_l] fp32 and [n] uint32, both required, copied (the buffers must stay valid until
 * the stream has passed this call).  Together with smtm_tables_import and smtm_hot_set this puts a saved
 * memory (centres, m, FT, TS, Psi) back so that inference and the memory update continue bit-identically. */
int32_t smtm_memory_import(smtm_ctx* ctx, int32_t exit, const float* centres_host,
                           const uint32_t* counts_host, void* stream);
/* Sets the fast memory Psi to k distinct class ids (host), hot_min <= k <= hot_max.  The ids are copied
 * before the call returns. */
int32_t smtm_hot_set(smtm_ctx* ctx, const int32_t* class_ids_host, int32_t k, void* stream);
/* Copies one exit point's centres ([n, C_l] fp32) and update counts ([n] uint32) to host
 * buffers (either may be NULL).  Synchronises the stream. */
int32_t smtm_memory_export(smtm_ctx* ctx, int32_t exit, float* centres_host, uint32_t* counts_host,
                           void* stream);
/* Copies the frequency table FT [n] and time-stamp table TS [n] (uint32), the fast-memory ids
 * in policy order (hot_ids_host sized hot_max) and the size k to host buffers (any may be
 * NULL).  Synchronises the stream. */
int32_t smtm_tables_export(smtm_ctx* ctx, uint32_t* ft_host, uint32_t* ts_host,
                           int32_t* hot_ids_host, int32_t* k_host, void* stream);
/* Overwrites FT and TS from host buffers [n] uint32 (either may be NULL = unchanged). */
int32_t smtm_tables_import(smtm_ctx* ctx, const uint32_t* ft_host, const uint32_t* ts_host,
                           void* stream);
/* Changes the threshold of Eq. 4 for the calls that follow. */
int32_t smtm_set_tau(smtm_ctx* ctx, float tau);

/* ---- one batch ----------------------------------------------------------------------------- */

/* Starts a batch of `batch` frames: SA := 0 (Eq. 3), all frames live, per-frame results cleared.
 * The call itself enqueues nothing: the batch's first smtm_encode / smtm_stage carries the initialisation in its
 * own kernel (one launch less per batch), and any other call that needs the batch's state enqueues it first. */
int32_t smtm_begin_batch(smtm_ctx* ctx, int32_t batch, void* stream);

/* 1. Encode (Sec. 4.1): semantic vector = mean over H x W of each channel, fp32 accumulation.
 *   fmap     device, NCHW contiguous [rows, C_l, H, W] of `dtype`, 16-byte aligned, read in place
 *   row_ids  device int32 or NULL.  NULL: slot i reads row i (a compacted tensor).  Otherwise
 *            slot i reads row row_ids[i]; smtm_live_ids() is the list to pass for a tensor
 *            that still holds the whole batch.  Rows must exist; they are not range-checked.
 *   sv_out   device [batch, C_l] fp32 or NULL: receives the semantic vectors by slot
 *            (rows of slots >= the live count are left untouched)
 * The number of live frames is read on the device. */
int32_t smtm_encode(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype,
                    int32_t H, int32_t W, const int32_t* row_ids, float* sv_out, void* stream);

/* Encode for channels-last feature maps: fmap is [rows, H, W, C_l] (NHWC), otherwise as
 * smtm_encode.  The semantic vectors are the same as for the NCHW tensor with the same values. */
int32_t smtm_encode_nhwc(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype,
                         int32_t H, int32_t W, const int32_t* row_ids, float* sv_out, void* stream);

/* 2. Lookup (Sec. 5 Steps 2-3, Sec. 6): for every live frame s_j = cos(SV, SC_j) for all n
 * classes (Eq. 1; 0 when either vector has zero or non-finite length), SA_j += 2^(exit-1) s_j
 * (Eq. 3), then highest / second-highest SA over the fast memory (tier 1) and over the global
 * memory (tier 2), ties ordered by (larger value, smaller class id), and the exit rule of
 * Eq. 4:  SA_H > 0  and  SA_H - SA_SH > tau * max(SA_SH, 0)   (= AC > tau when SA_SH > 0).
 * Tier 2 is consulted only when cfg.tiers == 2 and tier 1 did not release the frame.
 * Optional device outputs, by slot:
 *   top_val  [batch, 2 tiers, 2] fp32 {SA_H, SA_SH}      top_id  [batch, 2 tiers] int32 id of SA_H
 *   sims_out [batch, n] fp32  s_j of this exit point (for tests)
 * Requires smtm_encode for this exit point in this batch (else SMTM_ERR_STATE). */
int32_t smtm_lookup(smtm_ctx* ctx, int32_t exit, float* top_val, int32_t* top_id,
                    float* sims_out, void* stream);

/* Diagnostic, not on the decision path: single-layer separability (Eq. 2) of the live frames,
 * sep = (s_H - s_SH) / s_SH with s_H, s_SH the highest and second-highest similarity of THIS exit
 * point over the fast memory (tier 1) and over the global memory (tier 2).
 *   sims     device [batch, n] fp32: the sims_out of smtm_lookup for this exit point
 *   sep_out  device [batch, 2 tiers] fp32; +inf where s_SH <= 0 < s_H, -inf where s_H <= 0 or the
 *            tier has fewer than two entries
 * To be called after smtm_lookup and before smtm_exit_compact of the exit point (else SMTM_ERR_STATE). */
int32_t smtm_separability(smtm_ctx* ctx, int32_t exit, const float* sims, float* sep_out, void* stream);

/* 3. Exit and compact (Sec. 1 "skip the rest layers", Sec. 5 last paragraph): stable partition
 * of the live frames into those released at this exit point and those that continue.
 * Device outputs (any may be NULL), lists in ascending original frame id:
 *   exit_ids / exit_labels / exit_tier  [batch] int32, first n_exit entries valid
 *   n_exit_dev, n_live_dev              int32 scalars
 *   live_ids                            [batch] int32, first n_live entries valid
 * Optional gather of the survivors' feature maps into a dense tensor for the next block:
 *   fmap_in  the tensor given to smtm_encode at this exit point, with the same row_ids
 *   fmap_out device, [>= n_live rows] of row_bytes each, must not overlap fmap_in
 *   row_bytes bytes per frame (C*H*W*element size)
 * After the call the context's live list is the survivors' list.
 * Requires smtm_lookup for this exit point (else SMTM_ERR_STATE). */
int32_t smtm_exit_compact(smtm_ctx* ctx, int32_t exit,
                          int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                          int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev,
                          const void* fmap_in, const int32_t* row_ids, void* fmap_out,
                          int64_t row_bytes, void* stream);

/* 2 + 3 in one call, same results.  Arguments as in smtm_lookup (without sims_out) and
 * smtm_exit_compact.  Requires smtm_encode for this exit point (else SMTM_ERR_STATE). */
int32_t smtm_lookup_exit(smtm_ctx* ctx, int32_t exit, float* top_val, int32_t* top_id,
                         int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                         int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev,
                         const void* fmap_in, const int32_t* row_ids, void* fmap_out,
                         int64_t row_bytes, void* stream);

/* 1 + 2 + 3 for one exit point, same results. */
int32_t smtm_stage(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype,
                   int32_t H, int32_t W, const int32_t* row_ids,
                   int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                   int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev,
                   void* fmap_out, void* stream);
/* The same for a channels-last feature map [rows, H, W, C_l] (smtm_encode_nhwc in place of smtm_encode). */
int32_t smtm_stage_nhwc(smtm_ctx* ctx, int32_t exit, const void* fmap, int32_t dtype,
                        int32_t H, int32_t W, const int32_t* row_ids,
                        int32_t* exit_ids, int32_t* exit_labels, int32_t* exit_tier,
                        int32_t* n_exit_dev, int32_t* live_ids, int32_t* n_live_dev,
                        void* fmap_out, void* stream);

/* Name of the kernel instance that the last smtm_encode / smtm_encode_nhwc / smtm_stage of this exit point
 * launched (for reports; "" before the first encode).  The pointer stays valid until the next encode of
 * that exit point. */
const char* smtm_encode_kernel(const smtm_ctx* ctx, int32_t exit);

/* Device pointer to the context's current live list (original frame ids, ascending; the live
 * count is on the device, see smtm_read_counts).  Valid as row_ids for smtm_encode /
 * smtm_exit_compact / smtm_stage of the next exit point; it is overwritten two
 * smtm_exit_compact calls later. */
const int32_t* smtm_live_ids(const smtm_ctx* ctx);

/* Per-frame results of the batch so far, by original frame id, copied to device buffers
 * [batch] int32 (any may be NULL): exit_layer in 1..L or 0 (still live / ran to the end),
 * label (class of SA_H) or -1, tier 1 / 2 or 0. */
int32_t smtm_batch_results(smtm_ctx* ctx, int32_t* exit_layer, int32_t* label, int32_t* tier,
                           void* stream);

/* Copies the live count and the last exit count to host ints (either may be NULL).
 * Synchronises the stream. */
int32_t smtm_read_counts(smtm_ctx* ctx, int32_t* n_live_host, int32_t* n_exit_host, void* stream);

/* Per-exit-point counters of the current batch to host: [L][4] = live frames entering,
 * released by tier 1, released by tier 2, spare.  Synchronises the stream. */
int32_t smtm_read_stats(smtm_ctx* ctx, int32_t* stats_host, void* stream);

/* ---- between batches (Sec. 6) ------------------------------------------------------------- */

/* Memory update with the batch's outputs, frames taken in original order:
 *   label[b]      device int32 [batch]: recognised class or -1 (nothing recognised)
 *   stop_layer[b] device int32 [batch]: exit point at which inference stopped, 0 = do not
 *                 update centres with this frame.  Cut down to the exit points the frame has a saved
 *                 semantic vector for: the exit point at which the library released it, or, for a frame
 *                 that ran on, the exit points encoded in this batch
 *   Both NULL: the batch's own results are used (what smtm_batch_results would return: label
 *   and exit point of the frames released so far, -1 / 0 for the others).
 * (i)  FT_j += 1 for the frame's class, TS_i = consecutive frames without class i (Sec. 6.1);
 * (ii) centres of class label[b] at exit points 1..stop_layer[b] move to the running mean
 *      (SC*m + SV)/(m+1) with the semantic vectors saved by smtm_encode (Eq. 7);
 *      (with SMTM_FORGET_IN_PLACE the quartering is applied to FT_i as the frames go by instead);
 * (iii) Score_i = FT_i * 0.25^floor(TS_i/W) (Eq. 5, exact integers, exponent clamped at 15);
 * (iv) classes ordered by (Score desc, id asc); k = smallest size whose share of the total
 *      score reaches cl_num/cl_den (Eq. 6), clamped to [hot_min, hot_max]; the fast memory
 *      becomes the first k classes.  With no history (all scores 0) it is left as it is.
 * `batch` must equal the size given to smtm_begin_batch. */
int32_t smtm_cache_update(smtm_ctx* ctx, const int32_t* label, const int32_t* stop_layer,
                          int32_t batch, void* stream);

/* smtm_cache_update for callers that cannot allocate device memory or tolerate a library that does
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments,
 * same results, but the update's scratch (class histogram, last positions, scores, policy order, score
 * total, policy counter; 20 bytes per class) lives in an 82 KB array that is part of the library's
 * device image instead of in buffers allocated with the context.  The call itself allocates and frees nothing.
 *   - At most 4096 classes; a context with more gets SMTM_ERR_UNSUPPORTED and nothing is enqueued.
 *   - Every context on one GPU shares that GPU's array (each GPU has its own copy, held until the process
 *     ends).  Calls whose kernels may overlap on one GPU (two streams) race on it: order them.
 *   - Nothing is assumed about what an earlier call left in the array. */
int32_t smtm_cache_update_static(smtm_ctx* ctx, const int32_t* label, const int32_t* stop_layer,
                                 int32_t batch, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SMTM_H */
