// Device code shared by the lookup and the compaction kernels: the (value, id) top-2 order, the exit rule
// of Eq. 4 (arXiv 2112.02644) and the decision of one live frame from its per-tile partial results.
// Header-only because device functions are not linked across translation units here.
#pragma once

#include "internal.h"

namespace smtm {

constexpr int SC_FIELDS = 6;              // per frame and class tile: tier 1 {SA_H, id, SA_SH}, tier 2 the same

// ---------------------------------------------------------------------------------------------
// Top-2 bookkeeping.  The order is (larger value first, then smaller class id); id < 0 with value
// -inf marks "no entry".  Accumulated similarities are finite, so -inf never is a real entry.
// Everything is written with selects: as nested branches the per-element update costs several times
// the memory traffic of the row.
struct Top2 {
    float v1; int id1; float v2;
};

// One more entry for a running top-2 whose entries arrive in ascending id, so an equal value never
// displaces the best one (strict >).  `take` = false leaves the triple as it is.
__device__ __forceinline__ void top2_push(Top2& t, float v, int id, bool take = true) {
    const float x = take ? v : -__builtin_inff();
    const bool gt = x > t.v1;
    t.v2 = gt ? t.v1 : fmaxf(t.v2, x);
    t.id1 = gt ? id : t.id1;
    t.v1 = gt ? x : t.v1;
}

// Merge of another (best, id, second) triple; the second of a triple never exceeds its best.
__device__ __forceinline__ void top2_merge(Top2& t, float v1, int id1, float v2) {
    // ids compare as unsigned so that "no entry" (-1) loses a tie of two -inf against nothing real
    const bool b = (v1 > t.v1) | ((v1 == t.v1) & ((uint32_t)id1 < (uint32_t)t.id1));
    const float loser = b ? t.v1 : v1;
    t.v2 = fmaxf(fmaxf(t.v2, v2), loser);
    t.v1 = b ? v1 : t.v1;
    t.id1 = b ? id1 : t.id1;
}

__device__ __forceinline__ bool exit_rule(float h, float sh, float tau) {
    if (!(h > 0.f)) return false;
    if (sh == -__builtin_inff()) return false;           // fewer than two entries in the tier
    const float runner = sh > 0.f ? sh : 0.f;
    return (h - sh) > tau * runner;
}

// ---------------------------------------------------------------------------------------------
// Decision of one live slot from its per-tile partial results (Sec. 5 Step 3, Sec. 6 tiers, Eq. 4).
struct SlotTop2 {
    Top2 hot, all;
};

// Loads only: the slot's per-tile results merged in tile order.  Safe for any slot below part_stride (the
// buffer is allocated in full), so it can be issued before the live count is known.
__device__ __forceinline__ SlotTop2 merge_slot(const DecideArgs& g, int slot) {
    const float ninf = -__builtin_inff();
    SlotTop2 m = {{ninf, -1, ninf}, {ninf, -1, ninf}};
    const float* p = g.part + slot;
    const int64_t ps = g.part_stride;
    int t = 0;
    for (; t + 2 <= g.tiles; t += 2) {                   // two tiles (twelve loads) in flight
        float f[2][SC_FIELDS];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int k = 0; k < SC_FIELDS; ++k) f[u][k] = p[((int64_t)(t + u) * SC_FIELDS + k) * ps];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            top2_merge(m.hot, f[u][0], __builtin_bit_cast(int, f[u][1]), f[u][2]);
            top2_merge(m.all, f[u][3], __builtin_bit_cast(int, f[u][4]), f[u][5]);
        }
    }
    for (; t < g.tiles; ++t) {
        float f[SC_FIELDS];
#pragma unroll
        for (int k = 0; k < SC_FIELDS; ++k) f[k] = p[((int64_t)t * SC_FIELDS + k) * ps];
        top2_merge(m.hot, f[0], __builtin_bit_cast(int, f[1]), f[2]);
        top2_merge(m.all, f[3], __builtin_bit_cast(int, f[4]), f[5]);
    }
    return m;
}

// The exit rule on the merged values, and everything a live slot writes.
__device__ __forceinline__ SlotDecision finish_slot(const DecideArgs& g, int slot, SlotTop2 m) {
    const float ninf = -__builtin_inff();
    Top2& hot = m.hot;
    Top2& all = m.all;
    SlotDecision o;
    o.d = 0; o.label = -1;
    if (exit_rule(hot.v1, hot.v2, g.tau)) { o.d = 1; o.label = hot.id1; }
    else if (g.tiers == 2 && exit_rule(all.v1, all.v2, g.tau)) { o.d = 2; o.label = all.id1; }
    if (g.tiers != 2) { all.v1 = ninf; all.v2 = ninf; all.id1 = -1; }
    float* tv = g.top_val + (int64_t)slot * 4;
    tv[0] = hot.v1; tv[1] = hot.v2; tv[2] = all.v1; tv[3] = all.v2;
    g.top_id[slot * 2] = hot.id1; g.top_id[slot * 2 + 1] = all.id1;
    if (g.top_val_user) {
        float* u = g.top_val_user + (int64_t)slot * 4;
        u[0] = hot.v1; u[1] = hot.v2; u[2] = all.v1; u[3] = all.v2;
    }
    if (g.top_id_user) { g.top_id_user[slot * 2] = hot.id1; g.top_id_user[slot * 2 + 1] = all.id1; }
    g.decision[slot] = o.d;
    g.label[slot] = o.label;
    return o;
}

__device__ __forceinline__ SlotDecision decide_slot(const DecideArgs& g, int slot) {
    return finish_slot(g, slot, merge_slot(g, slot));
}

}  // namespace smtm
