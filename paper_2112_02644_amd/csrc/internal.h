// Internal declarations shared by the host runtime (api.hip) and the kernel files.
// Nothing here crosses the C ABI declared in include/smtm.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/smtm.h"

namespace smtm {

// Device-resident counters.  Kernels read the live count from here, so no launch ever waits
// for the host to learn how many frames are left.
struct Counts {
    int32_t n_live;                       // live frames entering the next exit point
    int32_t n_exit;                       // frames released by the last smtm_exit_compact
    int32_t hot_k;                        // current fast-memory size
    int32_t ticket;                       // spare
    int32_t stats[SMTM_MAX_EXITS][4];     // per exit point: live in, released tier 1, released tier 2, spare
};

struct CompactArgs {                      // everything the stable partition reads and writes
    const int32_t* decision;              // [slots] 0 continue, 1 / 2 released by tier 1 / 2
    const int32_t* label;                 // [slots]
    const int32_t* frame_ids;             // [slots] current live list
    int32_t* next_ids;                    // survivors' frame ids (the next live list)
    int32_t* next_slots;                  // survivors' old slots (for the row gather)
    Counts* counts;
    int max_rows;                         // entries in the lists above (the batch begun)
    int exit_index;                       // 1-based
    int32_t *exit_ids, *exit_labels, *exit_tier, *n_exit_dev, *live_ids_user, *n_live_dev;   // caller's, may be NULL
    int32_t *res_layer, *res_label, *res_tier;                                               // per-frame results
};

constexpr int kWave = 64;
constexpr int kRowMaxSlots = 64;          // partial maxima of |SV| kept per frame and exit point (one per bin of channel groups)
constexpr int kKPad = 64;                 // fp16 operand rows are zero-padded to a multiple of this many columns
constexpr int kRowPad = 128;              // fp16 operand matrices are padded to a multiple of this many rows

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Where element (class j, channel c) of the unit fp16 copy of the centres lives.  The copy is kept in the order
// the matrix cores take their B operand, so that a wavefront fetches the operand of one MFMA step (32 classes x
// 16 channels, 1 KB) with one fully contiguous load: [class tile of 32][step of 16 channels][lane][8 halves],
// where lane = 32 * (second half of the step's channels) + class within the tile.  Cp is a multiple of kKPad.
__host__ __device__ static inline int64_t chat_index(int j, int c, int Cp) {
    const int64_t step = (int64_t)(j >> 5) * (Cp >> 4) + (c >> 4);
    return ((step * 64) + ((c >> 3) & 1) * 32 + (j & 31)) * 8 + (c & 7);
}

// ---- encode.hip -------------------------------------------------------------------------
// Picks the streaming path from the shape; returns a short name of the path ("d16", "pair", "d8", "lds", "d4", "d2")
// and writes the name of the kernel instance it launched to `name` and the number of partial-maximum slots it fills
// per frame to `slots`.
struct EncodeOut {
    float* sv;                            // [max_rows, ldv] by live slot
    int ldv;
    int32_t* slot_of;                     // [frames] live slot of each frame at this exit point
    float* sv_out;                        // [max_rows, C] by slot, or NULL
    // Start of a batch folded into its first encode (saves a launch): fresh = batch size (0 = not the first encode).
    // The kernel then takes every frame as live in identity order instead of reading the count and the list, and
    // its threads also write what k_begin_batch would have written (list, per-frame results, counters).
    int fresh;
    int32_t* live0;                       // [batch] live list to initialise
    int32_t *res_layer, *res_label, *res_tier;
    Counts* counts_w;
    uint32_t* rowmax;                     // [max_rows, kRowMaxSlots] by live slot: largest |SV| (bit pattern) per bin of the frame's channel groups
};
const char* launch_encode(const void* fmap, int dtype, int C, int HW, const int32_t* row_ids,
                          const int32_t* frame_ids, const Counts* counts, int max_rows,
                          const EncodeOut& out, hipStream_t st, char* name, size_t name_cap, int* slots);

// Channels-last variant: fmap is [rows, H, W, C].
const char* launch_encode_nhwc(const void* fmap, int dtype, int C, int HW, const int32_t* row_ids,
                               const int32_t* frame_ids, const Counts* counts, int max_rows,
                               const EncodeOut& out, hipStream_t st, char* name, size_t name_cap, int* slots);

// ---- lookup.hip -------------------------------------------------------------------------
void launch_centre_prepare(const float* centres, int n, int C, float* cinv, _Float16* chat, int Cp,
                           int row_lo, int row_hi, hipStream_t st);

constexpr int kScoreTileRows = 32;        // live frames per scoring tile
constexpr int kScoreTileCols = 128;       // classes per scoring tile (= kRowPad)

struct ScoreArgs {
    const float* sv;                      // [max_rows, ldv] fp32 semantic vectors by live slot
    int ldv;                              // row stride of sv (channels rounded up to kKPad, zero padded)
    const uint32_t* rowmax;               // [max_rows, kRowMaxSlots] by live slot: partial maxima of |SV| (bit patterns)
    int rowmax_slots;                     // how many of a frame's slots the encode kernel filled
    const int32_t* frame_ids;             // [max_rows] live list
    const Counts* counts;
    int max_rows;
    int n;                                // classes
    float weight;                         // 2^(l-1)
    int first;                            // 1: first lookup of the batch, SA holds nothing yet: SA = weight * s
    float* SA;                            // [frames, n] by original frame id (with slack behind the last row)
    float* sims_out;                      // [max_rows, n] by slot, or NULL
    const uint8_t* in_hot;                // [n rounded up to kRowPad] fast-memory mask
    float* part;                          // [tiles][6][part_stride] per-tile best / second best by slot
    int part_stride;
};
void launch_score_mfma(const ScoreArgs& a, const _Float16* chat, int Cp, hipStream_t st);
void launch_score_fp32(const ScoreArgs& a, const float* centres, const float* cinv, int C, hipStream_t st);

struct DecideArgs {                       // merge of the per-tile results and the exit rule
    const float* part;
    int part_stride;
    int tiles;
    const Counts* counts;
    int max_rows;
    int tiers;
    float tau;
    int32_t* decision;                    // [max_rows] by slot: 0 continue, 1 / 2 released by tier 1 / 2
    int32_t* label;                       // [max_rows]
    float* top_val;                       // [max_rows, 2 tiers, 2]
    int32_t* top_id;                      // [max_rows, 2 tiers]
    float* top_val_user;                  // caller's copies, may be NULL
    int32_t* top_id_user;
};
struct SlotDecision {
    int d, label;
};
void launch_decide(const DecideArgs& g, hipStream_t st);

void launch_separability(const float* sims, const Counts* counts, int max_rows, int n, const uint8_t* in_hot,
                         float* sep_out, hipStream_t st);

// ---- compact.hip ------------------------------------------------------------------------
void launch_begin_batch(int batch, int32_t* live, int32_t* res_layer, int32_t* res_label, int32_t* res_tier,
                        Counts* counts, hipStream_t st);
void launch_compact(const CompactArgs& args, hipStream_t st);
void launch_decide_compact(const DecideArgs& g, const CompactArgs& args, hipStream_t st);
void launch_gather_rows(const void* src, const int32_t* row_ids, const int32_t* next_slots,
                        const Counts* counts, int max_rows, void* dst, int64_t row_bytes,
                        hipStream_t st);
void launch_copy3_i32(const int32_t* s0, int32_t* d0, const int32_t* s1, int32_t* d1, const int32_t* s2,
                      int32_t* d2, int count, hipStream_t st);
void launch_set_hot(const int32_t* ids, int k, int n, int32_t* hot_ids, uint8_t* in_hot, Counts* counts,
                    hipStream_t st);
void launch_fill_u32(uint32_t* dst, uint32_t value, int count, hipStream_t st);

// ---- update.hip -------------------------------------------------------------------------
struct CentreTables {                     // per exit point, passed by value to the centre-update kernel
    float* centres[SMTM_MAX_EXITS];
    uint32_t* mcount[SMTM_MAX_EXITS];
    float* cinv[SMTM_MAX_EXITS];
    _Float16* chat[SMTM_MAX_EXITS];
    const float* sv[SMTM_MAX_EXITS];      // [batch, Cp] saved semantic vectors by the live slot the frame had at that exit point
    const int32_t* slot_of[SMTM_MAX_EXITS];   // [batch] that slot, by original frame id (valid for frames live at the exit point)
    int C[SMTM_MAX_EXITS];
    int Cp[SMTM_MAX_EXITS];               // channels rounded up to kKPad: row stride of chat and of sv
    const int32_t* res_layer;             // [batch] exit point at which the library released the frame, 0 = not released
    int enc_upto;                         // exit points 1..enc_upto have been encoded in this batch
};
// The scratch arrays of one memory update (class histogram, last positions, scores, policy order, the
// 128-bit score total and the policy counter).
struct UpdateScratch {
    uint32_t* cls_cnt;
    int32_t* cls_last;
    uint64_t* score;
    int32_t* order;
    uint64_t* total;
    int32_t* below;
};
constexpr int kStaticMaxClasses = 4096;   // most classes the statically allocated update scratch is laid out for
// Device addresses of the statically allocated scratch on GPU `device`, which must be the current device.
hipError_t update_static_scratch(int device, UpdateScratch* out);

void launch_tables_update(const int32_t* label, int batch, int n, uint32_t W, uint32_t* FT, uint32_t* TS,
                          uint32_t* cls_cnt, int32_t* cls_last, uint64_t* score, uint64_t* total,
                          int32_t* below, int inplace, hipStream_t st);
void launch_class_count(const int32_t* label, int batch, int n, uint32_t* cls_cnt, hipStream_t st);
void launch_centres_update(const CentreTables& tabs, int n_exits, int n, const int32_t* label,
                           const int32_t* stop_layer, int batch, const uint32_t* cls_cnt, hipStream_t st);
void launch_centres_and_policy(const CentreTables& tabs, int n_exits, int n, const int32_t* label,
                               const int32_t* stop_layer, int batch, const uint32_t* cls_cnt,
                               const uint64_t* score, const uint64_t* total, uint32_t cl_num, uint32_t cl_den,
                               int hot_min, int hot_max, int32_t* order, int32_t* below, int32_t* hot_ids,
                               uint8_t* in_hot, Counts* counts, hipStream_t st);

}  // namespace smtm
