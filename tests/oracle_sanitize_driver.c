/*
 * Driver for the sanitizer run of the CPU oracle (tests/test_oracle_sanitizers.py): calls every
 * function of oracle/smtm_oracle.c on small inputs, edge cases included (no live frames, one
 * channel, ties, empty fast memory tier, saturated tables), so that AddressSanitizer and
 * UndefinedBehaviorSanitizer see every loop bound and every integer operation.  A few results are
 * checked against values that follow from the definitions; the exit status is 0 when all hold.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double orc_half_to_double(uint16_t h);
void orc_encode(const void *F, int dtype, int C, int HW, const int32_t *row_ids, int64_t n_live, double *SV);
double orc_cosine(const double *v, const double *c, int C);
double orc_cosine_abs_scale(const double *v, const double *c, int C);
double orc_weight(int l);
void orc_top2(const double *SA, const int32_t *ids, int count, double *SA_H, int32_t *id_H, double *SA_SH);
int orc_exit_predicate(double SA_H, double SA_SH, double tau);
double orc_accumulated_confidence(double SA_H, double SA_SH);
void orc_lookup(const double *SV, const double *SC, int n, int C, int l, const int32_t *frame_ids, int64_t n_live,
                double *SA, const int32_t *hot_ids, int k, int tiers, double tau, int32_t *decision, int32_t *label,
                double *top_val, int32_t *top_id, double *sims, double *sims_scale);
void orc_compact(const int32_t *decision, const int32_t *label, const int32_t *frame_ids, int64_t n_live,
                 int32_t *exit_ids, int32_t *exit_labels, int32_t *exit_tier, int32_t *n_exit,
                 int32_t *live_ids, int32_t *live_slots, int32_t *n_next);
void orc_tables_update(uint32_t *FT, uint32_t *TS, int n, const int32_t *label, int64_t batch);
void orc_tables_update_inplace(uint32_t *FT, uint32_t *TS, int n, uint32_t W, const int32_t *label, int64_t batch);
uint64_t orc_score_int(uint32_t FT, uint32_t TS, uint32_t W);
double orc_score_real(uint32_t FT, uint32_t TS, uint32_t W);
int32_t orc_select_hot(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W, uint32_t cl_num, uint32_t cl_den,
                       int32_t k_min, int32_t k_max, int32_t *order, int32_t *k_unclamped);
int32_t orc_select_hot_mode(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W, int inplace, uint32_t cl_num,
                            uint32_t cl_den, int32_t k_min, int32_t k_max, int32_t *order, int32_t *k_unclamped);
double orc_p_of_a(const uint32_t *FT, const uint32_t *TS, int n, uint32_t W, const int32_t *order, int k);
void orc_centres_update(double **SC, uint32_t **m, const int32_t *dims, int L, int n, double *const *SV,
                        const int32_t *label, const int32_t *stop_layer, int64_t batch);
void orc_warmup_centres(const double *SV, const int32_t *label, int64_t N, int n, int C, double *SC, uint32_t *m);
double orc_sep(double s_H, double s_SH);
double orc_separability(const double *s, const int32_t *ids, int count);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main(void)
{
    /* binary16: 1.0, -2.0, smallest subnormal, infinity */
    CHECK(orc_half_to_double(0x3c00) == 1.0 && orc_half_to_double(0xc000) == -2.0);
    CHECK(orc_half_to_double(0x0001) == ldexp(1.0, -24) && isinf(orc_half_to_double(0x7c00)));

    /* encode: 3 frames x 2 channels x 5 positions, fp32 and fp16, dense, through row ids, and with no live frame */
    enum { R = 3, C = 2, HW = 5 };
    float *F32 = malloc(sizeof(float) * R * C * HW);
    uint16_t *F16 = malloc(sizeof(uint16_t) * R * C * HW);
    for (int i = 0; i < R * C * HW; ++i) { F32[i] = (float)(i % 7) - 3.0f; F16[i] = 0x3c00; }
    double *SV = malloc(sizeof(double) * R * C);
    orc_encode(F32, 1, C, HW, NULL, R, SV);
    CHECK(fabs(SV[0] - (-3.0 - 2.0 - 1.0 + 0.0 + 1.0) / 5.0) < 1e-15);
    int32_t rows[2] = {2, 0};
    orc_encode(F16, 0, C, HW, rows, 2, SV);
    CHECK(SV[0] == 1.0 && SV[3] == 1.0);
    orc_encode(F16, 0, C, HW, rows, 0, SV);

    /* cosine and its tolerance scale, one channel included */
    double a[3] = {3.0, -4.0, 0.0}, b[3] = {4.0, 3.0, 0.0}, z[3] = {0.0, 0.0, 0.0};
    CHECK(orc_cosine(a, b, 3) == 0.0 && fabs(orc_cosine_abs_scale(a, b, 3) - 24.0 / 25.0) < 1e-15);
    CHECK(orc_cosine(a, a, 1) == 1.0 && orc_cosine(a, z, 3) == 0.0 && orc_cosine_abs_scale(z, b, 3) == 0.0);
    CHECK(orc_weight(1) == 1.0 && orc_weight(8) == 128.0);

    /* top-2: ties, a set of one, an empty set */
    double SA[5] = {0.5, 2.0, 2.0, -1.0, 0.25};
    double h, sh; int32_t id;
    orc_top2(SA, NULL, 5, &h, &id, &sh);
    CHECK(h == 2.0 && id == 1 && sh == 2.0);
    int32_t one[1] = {4};
    orc_top2(SA, one, 1, &h, &id, &sh);
    CHECK(h == 0.25 && id == 4 && isinf(sh) && sh < 0);
    orc_top2(SA, one, 0, &h, &id, &sh);
    CHECK(id == -1);
    CHECK(orc_exit_predicate(3.0, 1.0, 1.9) == 1 && orc_exit_predicate(3.0, 1.0, 2.0) == 0);
    CHECK(orc_exit_predicate(0.5, -0.5, 100.0) == 1 && orc_exit_predicate(-0.5, -0.75, 0.0) == 0);
    CHECK(orc_accumulated_confidence(3.0, 1.0) == 2.0 && isinf(orc_accumulated_confidence(1.0, 0.0)));

    /* lookup over two exit points, both tier settings, every optional output on and off */
    enum { N = 4, CC = 3, B = 3 };
    double SC[N * CC] = {1, 0, 0,  0, 1, 0,  0, 0, 1,  1, 1, 0};
    double V[B * CC] = {2, 0, 0,  0, 0, 0,  1, 1, 0.1};
    double *acc = calloc((size_t)B * N, sizeof(double));
    int32_t frames[B] = {0, 1, 2}, hot[2] = {3, 0};
    int32_t dec[B], lab[B], tid[B * 2];
    double tv[B * 4], sims[B * N], scale[B * N];
    /* frame 0 is class 0 exactly; in the fast memory {3, 0} the runner-up scores 1/sqrt(2): 1 - 0.707 > 0.25 * 0.707 */
    orc_lookup(V, SC, N, CC, 1, frames, B, acc, hot, 2, 2, 0.25, dec, lab, tv, tid, sims, scale);
    CHECK(dec[0] == 1 && lab[0] == 0 && dec[1] == 0 && lab[1] == -1);
    orc_lookup(V, SC, N, CC, 2, frames, B, acc, hot, 2, 1, 0.5, dec, lab, NULL, NULL, NULL, NULL);
    CHECK(fabs(acc[0] - 3.0) < 1e-15);                       /* 1 * 1 + 2 * 1 */
    orc_lookup(V, SC, N, CC, 3, frames, 0, acc, hot, 2, 2, 0.5, NULL, NULL, NULL, NULL, NULL, NULL);

    /* compaction: mixed, all leave, nobody leaves */
    int32_t ex_i[B], ex_l[B], ex_t[B], lv[B], ls[B], ne, nl;
    int32_t d1[B] = {1, 0, 2}, l1[B] = {7, -1, 9};
    orc_compact(d1, l1, frames, B, ex_i, ex_l, ex_t, &ne, lv, ls, &nl);
    CHECK(ne == 2 && nl == 1 && ex_i[1] == 2 && ex_t[1] == 2 && lv[0] == 1 && ls[0] == 1);
    int32_t d2[B] = {1, 1, 1}, d3[B] = {0, 0, 0};
    orc_compact(d2, l1, frames, B, ex_i, ex_l, ex_t, &ne, lv, NULL, &nl);
    CHECK(ne == 3 && nl == 0);
    orc_compact(d3, l1, frames, 0, ex_i, ex_l, ex_t, &ne, lv, ls, &nl);
    CHECK(ne == 0 && nl == 0);

    /* tables, saturation included, both forgetting modes */
    uint32_t FT[N] = {0, UINT32_MAX, 5, 0}, TS[N] = {0, UINT32_MAX - 1, 3, 0};
    int32_t labels[5] = {1, -1, 2, 1, 7};
    orc_tables_update(FT, TS, N, labels, 5);
    CHECK(FT[1] == UINT32_MAX && FT[2] == 6 && TS[2] == 2 && TS[0] == 5);
    uint32_t FT2[N] = {8, 8, UINT32_MAX, 1}, TS2[N] = {0, 1, UINT32_MAX, 0};
    orc_tables_update_inplace(FT2, TS2, N, 2, labels, 5);
    /* class 0 is quartered at TS = 2 and again at 4; class 2 restarts at its own frame and is quartered two frames later */
    CHECK(FT2[0] == 0 && FT2[1] == 3 && TS2[2] == 2 && FT2[2] == UINT32_MAX / 4);
    CHECK(orc_score_int(3, 0, 4) == ((uint64_t)3 << 30) && orc_score_int(3, 1000000, 4) == 3);
    CHECK(orc_score_real(16, 8, 4) == 1.0);
    int32_t order[N], ku;
    uint32_t FT3[N] = {1, 90, 5, 4}, TS3[N] = {0, 0, 0, 0};
    CHECK(orc_select_hot(FT3, TS3, N, 4, 19, 20, 1, N, order, &ku) == 2 && order[0] == 1 && order[1] == 2);
    CHECK(fabs(orc_p_of_a(FT3, TS3, N, 4, order, 2) - 0.95) < 1e-12);
    uint32_t zero[N] = {0, 0, 0, 0};
    CHECK(orc_select_hot_mode(zero, TS3, N, 4, 1, 19, 20, 1, N, order, &ku) == -1 && ku == -1);
    uint32_t big[N] = {UINT32_MAX, UINT32_MAX, UINT32_MAX, UINT32_MAX};
    CHECK(orc_select_hot(big, TS3, N, 4, 19, 20, 1, N, order, NULL) == 4);   /* 128-bit sums, no overflow */

    /* centres: two exit points, a frame that stops at each, one that updates nothing */
    int32_t dims[2] = {2, 1};
    double c0[N * 2] = {0}, c1[N] = {0};
    uint32_t m0[N] = {1, 1, 1, 1}, m1[N] = {0, 0, 0, 0};
    double *SCs[2] = {c0, c1};
    uint32_t *ms[2] = {m0, m1};
    double sv0[B * 2] = {2, 4,  6, 8,  1, 1}, sv1[B] = {5, 7, 9};
    double *SVs[2] = {sv0, sv1};
    int32_t ulab[B] = {2, 2, -1}, ustop[B] = {1, 2, 2};
    orc_centres_update(SCs, ms, dims, 2, N, SVs, ulab, ustop, B);
    CHECK(m0[2] == 3 && m1[2] == 1 && fabs(c0[4] - (0.0 + 2.0 + 6.0) / 3.0) < 1e-15 && c1[2] == 7.0);
    double wc[N * 2]; uint32_t wm[N];
    int32_t wl[B] = {3, 3, 9};
    orc_warmup_centres(sv0, wl, B, N, 2, wc, wm);
    CHECK(wm[3] == 2 && wc[6] == 4.0 && wc[7] == 6.0 && wm[0] == 0);
    CHECK(orc_sep(3.0, 1.0) == 2.0 && isinf(orc_separability(SA, one, 1)) && orc_separability(SA, NULL, 5) == 0.0);

    free(F32); free(F16); free(SV); free(acc);
    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    puts("oracle sanitizer driver: all checks hold");
    return 0;
}
