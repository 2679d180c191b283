/*
 * SMTM oracle — TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, double-precision CPU evaluation of the semantic-memory
 * inference path of "Boosting Mobile CNN Inference through Semantic Memory"
 * (arXiv 2112.02644).  It exists only so that the tests, the smoke check and
 * the benchmark's CPU-baseline leg have something independent to compare the
 * GPU library against.  It shares no code, header, table or helper with the
 * GPU library and must never be called from it.
 *
 * Every function evaluates a definition from the paper exactly as written,
 * one frame and one class at a time, with no blocking, fusion or reordering.
 * The only parallelism is an OpenMP loop over frames (frames are independent
 * in every definition used here).
 *
 * Notation follows the paper: SV^l semantic vector at exit point l (Sec. 4.1),
 * SC_j^l semantic centre of class j (Sec. 4.2), s_j^l cosine similarity
 * (Eq. 1), SA_j^l cumulative similarity (Eq. 3), AC^l accumulated confidence
 * (Eq. 4), FT / TS frequency and time-stamp tables and Score_i (Sec. 6.1,
 * Eq. 5), P(A) (Eq. 6), centre update (Eq. 7).
 *
 * Readings taken where the paper is silent are marked "reading:" below.
 *
 * Parity pins: every function here (orc_cosine_abs_scale included) is pinned by tests/test_oracle_*.py
 * against closed forms, library routines, invariants and brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_F16 0
#define ORC_F32 1

/* IEEE 754 binary16 -> double, by the format's definition:
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits. */
double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);            /* zero and subnormals: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

static double load_elem(const void *F, int dtype, int64_t idx)
{
    if (dtype == ORC_F16)
        return orc_half_to_double(((const uint16_t *)F)[idx]);
    return (double)((const float *)F)[idx];
}

/*
 * Sec. 4.1 (semantic vectors): global average pooling.  For a feature map of
 * C x H x W the semantic vector has C entries, each the average of one map.
 *
 *   F        NCHW contiguous, [*, C, H, W], fp16 or fp32
 *   row_ids  NULL: live frame i is row i of F; else it is row row_ids[i]
 *   SV       out, [n_live, C] double
 */
void orc_encode(const void *F, int dtype, int C, int HW,
                const int32_t *row_ids, int64_t n_live, double *SV)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_live; ++i) {
        int64_t row = row_ids ? row_ids[i] : i;
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            int64_t base = (row * C + c) * (int64_t)HW;
            for (int p = 0; p < HW; ++p)
                acc += load_elem(F, dtype, base + p);
            SV[i * C + c] = acc / (double)HW;
        }
    }
}

/*
 * Eq. 1: s_j = xi(SV, SC_j), the cosine of the angle between the two vectors.
 * reading: if either vector has zero or non-finite length the similarity is 0
 * (the paper does not discuss it; such a frame can then never match).
 */
double orc_cosine(const double *v, const double *c, int C)
{
    double dot = 0.0, vv = 0.0, cc = 0.0;
    for (int k = 0; k < C; ++k) {
        dot += v[k] * c[k];
        vv += v[k] * v[k];
        cc += c[k] * c[k];
    }
    double den = sqrt(vv) * sqrt(cc);
    if (!(den > 0.0) || !isfinite(den) || !isfinite(dot))
        return 0.0;
    return dot / den;
}

/* The scale of the rounding error of a dot product: sum |v_k||c_k| / (|v||c|).
 * Not part of the method; the tests use it to state the similarity tolerance. */
double orc_cosine_abs_scale(const double *v, const double *c, int C)
{
    double dot = 0.0, vv = 0.0, cc = 0.0;
    for (int k = 0; k < C; ++k) {
        dot += fabs(v[k] * c[k]);
        vv += v[k] * v[k];
        cc += c[k] * c[k];
    }
    double den = sqrt(vv) * sqrt(cc);
    if (!(den > 0.0) || !isfinite(den) || !isfinite(dot))
        return 0.0;
    return dot / den;
}

/* Sec. 5, Step 2: weight of exit point l (1-based) is 2^(l-1). */
double orc_weight(int l)
{
    return ldexp(1.0, l - 1);
}

/*
 * Highest and second-highest accumulated similarity over a set of classes
 * (Sec. 5, Step 3).  reading: ties are ordered by (larger value, then smaller
 * class id), whatever order the set is given in.
 *
 *   SA      [n] accumulated similarities of one frame
 *   ids     the set to search (class ids), or NULL for all of 0..n-1
 *   count   size of the set
 * Outputs id_H = -1 when the set is empty; SA_SH = -inf when it has < 2 members.
 */
void orc_top2(const double *SA, const int32_t *ids, int count,
              double *SA_H, int32_t *id_H, double *SA_SH)
{
    double best = -INFINITY, second = -INFINITY;
    int32_t best_id = -1, second_id = -1;
    for (int t = 0; t < count; ++t) {
        int32_t j = ids ? ids[t] : t;
        double x = SA[j];
        int beats_best = best_id < 0 || x > best || (x == best && j < best_id);
        if (beats_best) {
            second = best; second_id = best_id;
            best = x; best_id = j;
        } else {
            int beats_second = second_id < 0 || x > second || (x == second && j < second_id);
            if (beats_second) { second = x; second_id = j; }
        }
    }
    *SA_H = best; *id_H = best_id;
    *SA_SH = (second_id < 0) ? -INFINITY : second;
}

/*
 * Eq. 4 and the threshold rule below it: exit when AC = (SA_H - SA_SH)/SA_SH
 * exceeds tau (strictly).
 * reading: Eq. 4 is only meaningful for SA_SH > 0 (the paper's features are
 * post-ReLU, so its cosines are non-negative).  Multiplying through by a
 * positive SA_SH gives SA_H - SA_SH > tau * SA_SH; for SA_SH <= 0 < SA_H the
 * runner-up is not even positively correlated and the frame exits; for
 * SA_H <= 0 nothing matches and it never exits.  tau >= 0.
 */
int orc_exit_predicate(double SA_H, double SA_SH, double tau)
{
    if (!(SA_H > 0.0)) return 0;
    if (SA_SH == -INFINITY) return 0;            /* fewer than two entries: never exits */
    double runner = SA_SH > 0.0 ? SA_SH : 0.0;
    return (SA_H - SA_SH) > tau * runner;
}

/* Eq. 4 as printed, for reporting: +inf where SA_SH <= 0 < SA_H, -inf where SA_H <= 0. */
double orc_accumulated_confidence(double SA_H, double SA_SH)
{
    if (!(SA_H > 0.0)) return -INFINITY;
    if (!(SA_SH > 0.0)) return INFINITY;
    return (SA_H - SA_SH) / SA_SH;
}

/*
 * One exit point for a set of live frames: Sec. 5 Steps 2 and 3 with the
 * hierarchical memory of Sec. 6 (fast memory Psi first; reading: when
 * tiers == 2 a frame that the fast memory does not release is then matched
 * against the whole global memory Phi; tiers == 1 is the paper's
 * fast-memory-only lookup).
 *
 *   SV        [n_live, C]   semantic vectors of the live frames (orc_encode)
 *   SC        [n, C]        semantic centres of this exit point
 *   l         exit point, 1-based
 *   frame_ids [n_live]      original frame id of each live frame (row of SA)
 *   SA        [*, n]        in/out, accumulated similarities by ORIGINAL frame id
 *   hot_ids   [k]           the fast memory Psi
 * Outputs, all [n_live] unless stated (any may be NULL):
 *   decision  0 = continues, 1 = exits on fast memory, 2 = exits on global memory
 *   label     class id of SA_H of the tier that released it, else -1
 *   top_val   [n_live, 2, 2] (tier, {SA_H, SA_SH});  top_id [n_live, 2]
 *   sims      [n_live, n]   s_j^l
 *   sims_scale[n_live, n]   rounding-error scale of s_j^l (orc_cosine_abs_scale)
 */
void orc_lookup(const double *SV, const double *SC, int n, int C, int l,
                const int32_t *frame_ids, int64_t n_live, double *SA,
                const int32_t *hot_ids, int k, int tiers, double tau,
                int32_t *decision, int32_t *label,
                double *top_val, int32_t *top_id, double *sims, double *sims_scale)
{
    double w = orc_weight(l);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_live; ++i) {
        const double *v = SV + i * C;
        double *sa = SA + (int64_t)frame_ids[i] * n;
        for (int j = 0; j < n; ++j) {
            double s = orc_cosine(v, SC + (int64_t)j * C, C);
            if (sims) sims[i * n + j] = s;
            if (sims_scale) sims_scale[i * n + j] = orc_cosine_abs_scale(v, SC + (int64_t)j * C, C);
            sa[j] += s * w;                       /* Eq. 3 */
        }
        double h1, sh1, h2 = -INFINITY, sh2 = -INFINITY;
        int32_t id1, id2 = -1;
        int d = 0, lab = -1;
        orc_top2(sa, hot_ids, k, &h1, &id1, &sh1);
        if (orc_exit_predicate(h1, sh1, tau)) { d = 1; lab = id1; }
        if (tiers == 2) {
            orc_top2(sa, NULL, n, &h2, &id2, &sh2);
            if (d == 0 && orc_exit_predicate(h2, sh2, tau)) { d = 2; lab = id2; }
        }
        if (decision) decision[i] = d;
        if (label) label[i] = lab;
        if (top_val) {
            top_val[i * 4 + 0] = h1; top_val[i * 4 + 1] = sh1;
            top_val[i * 4 + 2] = h2; top_val[i * 4 + 3] = sh2;
        }
        if (top_id) { top_id[i * 2 + 0] = id1; top_id[i * 2 + 1] = id2; }
    }
}

/*
 * Skipping the remaining layers (Sec. 1 "Our proposal", Sec. 5 last
 * paragraph) for a batch: frames that exit leave, the others continue, both
 * lists kept in ascending original frame order.
 */
void orc_compact(const int32_t *decision, const int32_t *label, const int32_t *frame_ids,
                 int64_t n_live,
                 int32_t *exit_ids, int32_t *exit_labels, int32_t *exit_tier, int32_t *n_exit,
                 int32_t *live_ids, int32_t *live_slots, int32_t *n_next)
{
    int32_t ne = 0, nl = 0;
    for (int64_t i = 0; i < n_live; ++i) {
        if (decision[i] != 0) {
            exit_ids[ne] = frame_ids[i];
            exit_labels[ne] = label[i];
            exit_tier[ne] = decision[i];
            ++ne;
        } else {
            live_ids[nl] = frame_ids[i];
            if (live_slots) live_slots[nl] = (int32_t)i;
            ++nl;
        }
    }
    *n_exit = ne; *n_next = nl;
}

/*
 * Sec. 6.1, frequency table and time-stamp table, frame by frame in the
 * order the frames were seen: FT_i counts appearances of class i; TS_i is
 * the number of consecutive frames in which class i has not appeared.
 * reading: a frame whose label is -1 (nothing recognised) advances every
 * TS_i and touches no FT_i.  Both tables saturate at 2^32 - 1.
 */
void orc_tables_update(uint32_t *FT, uint32_t *TS, int n, const int32_t *label, int64_t batch)
{
    for (int64_t b = 0; b < batch; ++b) {
        for (int i = 0; i < n; ++i)
            if (TS[i] != UINT32_MAX) TS[i] += 1;
        int32_t j = label[b];
        if (j >= 0 && j < n) {
            TS[j] = 0;
            if (FT[j] != UINT32_MAX) FT[j] += 1;
        }
    }
}

/*
 * Sec. 6.1, forgetting applied in place (the variant the text gives before Eq. 5 and Sec. 8.1 uses
 * for fast-changing scenes): "we decay the memory ... every consecutive W frames".  Frame by frame:
 * for every class other than the frame's own, TS_i += 1 and, each time TS_i reaches a multiple of
 * W, the frequency entry is multiplied by 0.25; the frame's own class gets TS = 0, FT += 1.
 * reading: the frequency entry is an integer count and 0.25 x is floor(x / 4).
 */
void orc_tables_update_inplace(uint32_t *FT, uint32_t *TS, int n, uint32_t W,
                               const int32_t *label, int64_t batch)
{
    for (int64_t b = 0; b < batch; ++b) {
        int32_t j = label[b];
        for (int i = 0; i < n; ++i) {
            if (i == j) continue;
            if (TS[i] != UINT32_MAX) {
                TS[i] += 1;
                if (TS[i] % W == 0) FT[i] /= 4;
            }
        }
        if (j >= 0 && j < n) {
            TS[j] = 0;
            if (FT[j] != UINT32_MAX) FT[j] += 1;
        }
    }
}

/*
 * Eq. 5 in exact integer arithmetic.  Score_i = FT_i * 0.25^floor(TS_i / W).
 * reading: the exponent q is clamped at 15 and every score is scaled by the
 * common factor 4^15, which changes neither the order nor the ratio of
 * Eq. 6:  ScoreInt_i = FT_i * 4^(15 - q).
 */
#define ORC_QMAX 15
uint64_t orc_score_int(uint32_t FT, uint32_t TS, uint32_t W)
{
    uint32_t q = TS / W;
    if (q > ORC_QMAX) q = ORC_QMAX;
    return (uint64_t)FT << (2 * (ORC_QMAX - q));
}

/* Eq. 5 as printed, in floating point (reporting / pin against the integer form). */
double orc_score_real(uint32_t FT, uint32_t TS, uint32_t W)
{
    return (double)FT * pow(0.25, floor((double)TS / (double)W));
}

/*
 * Sec. 6.1 replacement policy and Sec. 6.2 adaptive cache size (Eq. 6).
 * Classes are ordered by (Score descending, class id ascending); P(A) for a
 * cache of the first k of them is the sum of their scores over the sum of all
 * scores.  reading: the cache size is the smallest k whose P(A) reaches the
 * confidence level CL = cl_num / cl_den (>=), clamped to [k_min, k_max];
 * with no history (all scores 0) the previous fast memory is kept.
 *
 *   order   out [n]  class ids in policy order
 *   returns the new k (or -1 when all scores are 0: caller keeps the old set)
 */
typedef struct { uint64_t score; int32_t id; } orc_entry;

static int cmp_entry(const void *a, const void *b)
{
    const orc_entry *x = (const orc_entry *)a, *y = (const orc_entry *)b;
    if (x->score != y->score) return x->score > y->score ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}

int32_t orc_select_hot_mode(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W, int inplace,
                            uint32_t cl_num, uint32_t cl_den, int32_t k_min, int32_t k_max,
                            int32_t *order, int32_t *k_unclamped);

int32_t orc_select_hot(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W,
                       uint32_t cl_num, uint32_t cl_den, int32_t k_min, int32_t k_max,
                       int32_t *order, int32_t *k_unclamped)
{
    return orc_select_hot_mode(FT, TS, n, W, 0, cl_num, cl_den, k_min, k_max, order, k_unclamped);
}

/* inplace != 0: the forgetting has already been applied to FT, so Score_i = FT_i. */
int32_t orc_select_hot_mode(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W, int inplace,
                            uint32_t cl_num, uint32_t cl_den, int32_t k_min, int32_t k_max,
                            int32_t *order, int32_t *k_unclamped)
{
    orc_entry *e = (orc_entry *)malloc(sizeof(orc_entry) * (size_t)n);
    unsigned __int128 total = 0;
    for (int i = 0; i < n; ++i) {
        e[i].score = inplace ? (uint64_t)FT[i] : orc_score_int(FT[i], TS[i], W);
        e[i].id = i;
        total += e[i].score;
    }
    qsort(e, (size_t)n, sizeof(orc_entry), cmp_entry);
    for (int i = 0; i < n; ++i) order[i] = e[i].id;
    int32_t k = -1;
    if (total != 0) {
        unsigned __int128 part = 0;
        for (int i = 0; i < n; ++i) {
            part += e[i].score;
            if (part * cl_den >= total * cl_num) { k = i + 1; break; }
        }
        if (k_unclamped) *k_unclamped = k;
        if (k < k_min) k = k_min;
        if (k > k_max) k = k_max;
    } else if (k_unclamped) {
        *k_unclamped = -1;
    }
    free(e);
    return k;
}

/* Eq. 6 as printed: P(A) for the first k classes of the policy order, in double. */
double orc_p_of_a(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W,
                  const int32_t *order, int k)
{
    double total = 0.0, part = 0.0;
    for (int i = 0; i < n; ++i) total += (double)orc_score_int(FT[i], TS[i], W);
    for (int i = 0; i < k; ++i) part += (double)orc_score_int(FT[order[i]], TS[order[i]], W);
    return total > 0.0 ? part / total : 0.0;
}

/*
 * Eq. 7, adaptive semantic centres, frame by frame in the order seen: if the
 * prediction for the frame is class j and inference stopped at exit point l,
 * then for every l0 in [1, l]:  SC' = (SC * m + SV) / (m + 1),  m' = m + 1.
 * reading: the range is inclusive of l (the equation), frames with label < 0
 * or stop_layer == 0 update nothing.
 *
 *   SC[l0]   [n, C_l0] double, in/out      m[l0]  [n] update counts, in/out
 *   SV[l0]   [batch, C_l0] double, semantic vector of each frame by ORIGINAL id
 *            (rows of frames that did not reach l0 are never read)
 */
void orc_centres_update(double **SC, uint32_t **m, const int32_t *dims, int L, int n,
                        double *const *SV, const int32_t *label, const int32_t *stop_layer,
                        int64_t batch)
{
    for (int64_t b = 0; b < batch; ++b) {
        int32_t j = label[b], l = stop_layer[b];
        if (j < 0 || j >= n || l < 1) continue;
        if (l > L) l = L;
        for (int l0 = 1; l0 <= l; ++l0) {
            int C = dims[l0 - 1];
            double *sc = SC[l0 - 1] + (int64_t)j * C;
            const double *sv = SV[l0 - 1] + b * C;
            double mm = (double)m[l0 - 1][j];
            for (int c = 0; c < C; ++c)
                sc[c] = (sc[c] * mm + sv[c]) / (mm + 1.0);
            m[l0 - 1][j] += 1;
        }
    }
}

/*
 * Sec. 5 / Sec. 6.3, warm-up: the semantic centre of a class is the average of the semantic
 * vectors of its training samples, and its update count m is the number of those samples.
 *
 *   SV     [N, C] semantic vectors of the training frames (one exit point)
 *   label  [N] class of each frame (frames with label outside 0..n-1 are ignored)
 *   SC     out [n, C]; a class without samples gets the zero vector and m = 0
 */
void orc_warmup_centres(const double *SV, const int32_t *label, int64_t N, int n, int C,
                        double *SC, uint32_t *m)
{
    for (int j = 0; j < n; ++j) {
        m[j] = 0;
        for (int c = 0; c < C; ++c) SC[(int64_t)j * C + c] = 0.0;
    }
    for (int64_t b = 0; b < N; ++b) {
        int32_t j = label[b];
        if (j < 0 || j >= n) continue;
        m[j] += 1;
        for (int c = 0; c < C; ++c) SC[(int64_t)j * C + c] += SV[b * C + c];
    }
    for (int j = 0; j < n; ++j)
        if (m[j] > 0)
            for (int c = 0; c < C; ++c) SC[(int64_t)j * C + c] /= (double)m[j];
}

/* Eq. 2 (single-layer separability), for diagnostics only. */
double orc_sep(double s_H, double s_SH)
{
    return (s_H - s_SH) / s_SH;
}

/*
 * Eq. 2 for one frame over a set of classes: s_H and s_SH are the highest and second-highest
 * similarity of one exit point.  reading (as for Eq. 4): +inf where s_SH <= 0 < s_H, -inf where
 * s_H <= 0 or the set has fewer than two members.
 */
double orc_separability(const double *s, const int32_t *ids, int count)
{
    double h, sh;
    int32_t id;
    orc_top2(s, ids, count, &h, &id, &sh);
    if (!(h > 0.0) || sh == -INFINITY) return -INFINITY;
    if (!(sh > 0.0)) return INFINITY;
    return orc_sep(h, sh);
}
