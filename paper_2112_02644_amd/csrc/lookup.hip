// Lookup: cosine similarity of every live frame's semantic vector with every class centre
// (arXiv 2112.02644, Eq. 1), accumulation over exit points with weight 2^(l-1) (Eq. 3), and per
// memory tier the highest / second-highest accumulated similarity with the exit rule of Eq. 4.
//
// Everything read here (semantic vectors, centres, SA) is a few MB and stays in L2; the only
// dense contraction is [live frames] x [classes] x [channels], which runs on the matrix cores
// with unit-normalised fp16 operands and fp32 accumulation, or in fp32 vector arithmetic when
// the feature maps are fp32.
#include "internal.h"

namespace smtm {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float x) {
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ float inv_norm_of(float nrm2) {
    // 0 marks a vector with zero or non-finite length: its similarities are defined as 0.
    if (!(nrm2 > 0.f) || !(nrm2 < __builtin_inff())) return 0.f;
    return 1.0f / sqrtf(nrm2);
}

// One wavefront per class: 1/|SC_j| and the unit-normalised fp16 copy [n_pad, Cp] (zero padded).
__global__ __launch_bounds__(256) void k_centre_prepare(const float* __restrict__ centres, int n, int C,
                                                        float* __restrict__ cinv,
                                                        _Float16* __restrict__ chat, int Cp,
                                                        int row_lo, int row_hi) {
    const int lane = threadIdx.x & 63;
    const int j = row_lo + blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= row_hi) return;
    if (j >= n) {                                       // padding rows of the fp16 copy
        for (int c = lane; c < Cp; c += 64) chat[(int64_t)j * Cp + c] = (_Float16)0.f;
        return;
    }
    const float* p = centres + (int64_t)j * C;
    float ss = 0.f;
    for (int c = lane; c < C; c += 64) { const float x = p[c]; ss += x * x; }
    ss = wave_sum(ss);
    const float inv = inv_norm_of(ss);
    if (lane == 0) cinv[j] = inv;
    for (int c = lane; c < Cp; c += 64) {
        float x = 0.f;
        if (c < C && inv != 0.f) x = p[c] * inv;
        chat[(int64_t)j * Cp + c] = (_Float16)x;
    }
}

void launch_centre_prepare(const float* centres, int n, int C, float* cinv, _Float16* chat, int Cp,
                           int row_lo, int row_hi, hipStream_t st) {
    const int rows = row_hi - row_lo;
    if (rows <= 0) return;
    hipLaunchKernelGGL(k_centre_prepare, dim3((rows + 3) / 4), dim3(256), 0, st, centres, n, C, cinv,
                       chat, Cp, row_lo, row_hi);
}

// One wavefront per live slot: 1/|SV| and (optionally) the unit-normalised fp16 row for the MFMA
// path.  The row is read with 16-byte loads, four per lane in flight, when C is a multiple of 4.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_rownorm(const float* __restrict__ sv,
                                                 const int32_t* __restrict__ frame_ids,
                                                 const Counts* __restrict__ counts, int max_rows, int C,
                                                 float* __restrict__ vinv, _Float16* __restrict__ vhat,
                                                 int Cp) {
    const int lane = threadIdx.x & 63;
    int slot = blockIdx.x * 4 + (threadIdx.x >> 6);
    // The first slot's frame id is fetched together with the live count: both come from memory written by
    // the kernel before, and one after the other they would cost two round trips.  The list has max_rows
    // entries, all of them frame ids of this or an earlier batch.
    int n_live = counts->n_live;
    int fid = slot < max_rows ? frame_ids[slot] : 0;
    asm volatile("" : "+v"(fid), "+s"(n_live));          // both loads are issued before either is waited for
    if (n_live > max_rows) n_live = max_rows;
    const int n_waves = gridDim.x * 4;
    const bool vec = (C & 3) == 0;
    for (; slot < n_live; slot += n_waves, fid = slot < n_live ? frame_ids[slot] : 0) {
        const float* p = sv + (int64_t)fid * C;
        float ss = 0.f;
        if (vec && Cp <= 2048) {
            // the row stays in registers between the norm and the fp16 copy (at most 8 x 16 bytes per lane)
            const f32x4* p4 = reinterpret_cast<const f32x4*>(p);
            const int nq = C >> 2, nqp = Cp >> 2;           // Cp is a multiple of 64
            f32x4 x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = u * 64 + lane;
                x[u] = q < nq ? p4[q] : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                ss += (x[u].x * x[u].x + x[u].y * x[u].y) + (x[u].z * x[u].z + x[u].w * x[u].w);
            ss = wave_sum(ss);
            const float inv = inv_norm_of(ss);
            if (lane == 0) vinv[slot] = inv;
            if (vhat) {
                _Float16* out = vhat + (int64_t)slot * Cp;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int q = u * 64 + lane;
                    if (q < nqp) {
                        f32x4 y = {0.f, 0.f, 0.f, 0.f};     // a zero or non-finite row (inv = 0) becomes zeros, as the padding
                        if (inv != 0.f) y = x[u] * inv;
                        const half4_t h = {(_Float16)y.x, (_Float16)y.y, (_Float16)y.z, (_Float16)y.w};
                        *reinterpret_cast<half4_t*>(out + 4 * q) = h;
                    }
                }
            }
            continue;
        }
        if (vec) {
            const f32x4* p4 = reinterpret_cast<const f32x4*>(p);
            const int nq = C >> 2;
            for (int base = 0; base < nq; base += 256) {
                f32x4 x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = base + u * 64 + lane;
                    x[u] = q < nq ? p4[q] : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    ss += (x[u].x * x[u].x + x[u].y * x[u].y) + (x[u].z * x[u].z + x[u].w * x[u].w);
            }
        } else {
            for (int c = lane; c < C; c += 64) { const float x = p[c]; ss += x * x; }
        }
        ss = wave_sum(ss);
        const float inv = inv_norm_of(ss);
        if (lane == 0) vinv[slot] = inv;
        if (vhat) {
            _Float16* out = vhat + (int64_t)slot * Cp;
            if (vec) {
                const f32x4* p4 = reinterpret_cast<const f32x4*>(p);
                const int nq = C >> 2, nqp = Cp >> 2;       // Cp is a multiple of 64
                for (int q = lane; q < nqp; q += 64) {
                    f32x4 x = {0.f, 0.f, 0.f, 0.f};
                    if (q < nq && inv != 0.f) x = p4[q] * inv;
                    half4_t h = {(_Float16)x.x, (_Float16)x.y, (_Float16)x.z, (_Float16)x.w};
                    *reinterpret_cast<half4_t*>(out + 4 * q) = h;
                }
            } else {
                for (int c = lane; c < Cp; c += 64) {
                    float x = 0.f;
                    if (c < C && inv != 0.f) x = p[c] * inv;
                    out[c] = (_Float16)x;
                }
            }
        }
    }
}

void launch_rownorm(const float* sv, const int32_t* frame_ids, const Counts* counts, int max_rows,
                    int C, float* vinv, _Float16* vhat, int Cp, hipStream_t st) {
    int grid = (max_rows + 3) / 4;
    if (grid > 2048) grid = 2048;
    hipLaunchKernelGGL(k_rownorm, dim3(grid), dim3(256), 0, st, sv, frame_ids, counts, max_rows, C, vinv,
                       vhat, Cp);
}

// ---------------------------------------------------------------------------------------------
// fp32 scoring: 64 slots x 64 classes per block, 4 x 4 per thread, K staged through LDS.
// s = <SV, SC_j> * (1/|SV|) * (1/|SC_j|);  SA[frame][j] += weight * s.
constexpr int FT_M = 64, FT_N = 64, FT_K = 16;

__global__ __launch_bounds__(256) void k_score_fp32(
    const float* __restrict__ sv, const int32_t* __restrict__ frame_ids,
    const Counts* __restrict__ counts, int max_rows, const float* __restrict__ vinv,
    const float* __restrict__ centres, const float* __restrict__ cinv, int n, int C, float weight,
    float* __restrict__ SA, float* __restrict__ sims_out) {
    __shared__ float As[FT_K][FT_M + 4];
    __shared__ float Bs[FT_K][FT_N + 4];
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int m0 = blockIdx.y * FT_M, n0 = blockIdx.x * FT_N;
    if (m0 >= n_live) return;                            // uniform over the block
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int lr = tid >> 2, lk = (tid & 3) * 4;         // loader: row 0..63, k offset 0,4,8,12
    const int a_slot = m0 + lr, b_cls = n0 + lr;
    const float* a_ptr = a_slot < n_live ? sv + (int64_t)frame_ids[a_slot] * C : nullptr;
    const float* b_ptr = b_cls < n ? centres + (int64_t)b_cls * C : nullptr;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < C; k0 += FT_K) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = k0 + lk + i;
            As[lk + i][lr] = (a_ptr && k < C) ? a_ptr[k] : 0.f;
            Bs[lk + i][lr] = (b_ptr && k < C) ? b_ptr[k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FT_K; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int slot = m0 + ty * 4 + i;
        if (slot >= n_live) continue;
        const float vi = vinv[slot];
        const int64_t frame = frame_ids[slot];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int cls = n0 + tx * 4 + j;
            if (cls >= n) continue;
            const float ci = cinv[cls];
            float s = acc[i][j] * vi * ci;
            if (vi == 0.f || ci == 0.f || !(fabsf(s) < __builtin_inff())) s = 0.f;
            SA[frame * n + cls] += weight * s;
            if (sims_out) sims_out[(int64_t)slot * n + cls] = s;
        }
    }
}

void launch_score_fp32(const float* sv, const int32_t* frame_ids, const Counts* counts, int max_rows,
                       const float* vinv, const float* centres, const float* cinv, int n, int C,
                       float weight, float* SA, float* sims_out, hipStream_t st) {
    dim3 grid((n + FT_N - 1) / FT_N, (max_rows + FT_M - 1) / FT_M);
    hipLaunchKernelGGL(k_score_fp32, grid, dim3(256), 0, st, sv, frame_ids, counts, max_rows, vinv,
                       centres, cinv, n, C, weight, SA, sims_out);
}

// ---------------------------------------------------------------------------------------------
// MFMA scoring.  A = unit fp16 semantic vectors by slot [rows_pad, Cp], B = unit fp16 centres
// [n_pad, Cp], both K-contiguous and zero padded, so S = A * B^T needs no bounds checks inside
// the K loop.  Block = 4 wavefronts as 2 x 2, each wavefront one 32x32 tile per (WM, WN) repeat,
// v_mfma_f32_32x32x16_f16: lane holds A[row = lane%32][k = 8*(lane/32) .. +7] and the same for
// B by column; acc[i] is C[row = 8*(i/4) + 4*(lane/32) + i%4][col = lane%32].
constexpr int MF_K = 64;                 // K per LDS stage
constexpr int MF_LD = MF_K + 8;          // padded LDS row (halves): 144 B keeps 16-byte reads conflict-free

template <int WM, int WN>
__global__ __launch_bounds__(256) void k_score_mfma(
    const _Float16* __restrict__ A, const _Float16* __restrict__ B, int Cp,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows, int n,
    float weight, float* __restrict__ SA, float* __restrict__ sims_out) {
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int RA = BM / 32, RB = BN / 32;            // 16-byte chunks each thread moves per stage
    __shared__ _Float16 As[2][BM * MF_LD];               // double buffered: the next K stage is fetched
    __shared__ _Float16 Bs[2][BN * MF_LD];               // from L2 while the current one is multiplied
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lk = (lane >> 5) * 8;

    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // loader: each 64-half row of a stage is 8 chunks of 16 B; thread -> (row, chunk)
    const int ld_row = tid >> 3, ld_chunk = tid & 7;
    const _Float16* a_src = A + (int64_t)(m0 + ld_row) * Cp + ld_chunk * 8;
    const _Float16* b_src = B + (int64_t)(n0 + ld_row) * Cp + ld_chunk * 8;
    const int lds_off = ld_row * MF_LD + ld_chunk * 8;
    // Four register sets: while stage st is multiplied out of LDS, the loads of stages st+2 .. st+4 are
    // in flight and stage st+1 (loaded three iterations earlier) is written to the other LDS buffer.
    // A stage is 16 KB per block from L2 or beyond; with fewer stages in flight the K loop runs at the
    // pace of that latency.
    u32x4 ra0[RA], rb0[RB], ra1[RA], rb1[RB], ra2[RA], rb2[RB], ra3[RA], rb3[RB];
    const int n_stage = Cp / MF_K;
    auto fetch = [&](u32x4* ra, u32x4* rb, int stage) {
        const int k1 = stage * MF_K;
#pragma unroll
        for (int r = 0; r < RA; ++r) ra[r] = *reinterpret_cast<const u32x4*>(a_src + (int64_t)r * 32 * Cp + k1);
#pragma unroll
        for (int r = 0; r < RB; ++r) rb[r] = *reinterpret_cast<const u32x4*>(b_src + (int64_t)r * 32 * Cp + k1);
    };
    auto stash = [&](const u32x4* ra, const u32x4* rb, int buf) {
#pragma unroll
        for (int r = 0; r < RA; ++r) *reinterpret_cast<u32x4*>(&As[buf][lds_off + r * 32 * MF_LD]) = ra[r];
#pragma unroll
        for (int r = 0; r < RB; ++r) *reinterpret_cast<u32x4*>(&Bs[buf][lds_off + r * 32 * MF_LD]) = rb[r];
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < MF_K; ks += 16) {
            half8_t a[WM], b[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i)
                a[i] = *reinterpret_cast<const half8_t*>(&As[buf][((wm * WM + i) * 32 + lrow) * MF_LD + ks + lk]);
#pragma unroll
            for (int j = 0; j < WN; ++j)
                b[j] = *reinterpret_cast<const half8_t*>(&Bs[buf][((wn * WN + j) * 32 + lrow) * MF_LD + ks + lk]);
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };
    // the operand loads are in bounds whatever the live count is (padded matrices), so they are
    // issued before the live count is waited for
    fetch(ra0, rb0, 0);
    if (n_stage > 1) fetch(ra1, rb1, 1);
    if (n_stage > 2) fetch(ra2, rb2, 2);
    if (n_stage > 3) fetch(ra3, rb3, 3);
    // Frame ids of this thread's output rows, then the old SA values of its outputs: two batches of
    // loads (all ids, then all values) that complete under the K loop.  Indices are clamped into the
    // buffers so that no load sits behind a branch (one behind a branch waits for the one before it,
    // and sixteen such pairs in a row cost more than the whole contraction); the list holds max_rows
    // frame ids of this or an earlier batch, so every address is inside SA, and what is fetched for
    // rows or classes outside the live tile is never used.
    int fid[WM][16];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int slot = m0 + (wm * WM + i) * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            fid[i][e] = frame_ids[slot < max_rows ? slot : max_rows - 1];
        }
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    if (m0 >= n_live) return;                            // uniform over the block
    stash(ra0, rb0, 0);
    __syncthreads();

    float sa_old[WM][WN][16];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int cls = n0 + (wn * WN + j) * 32 + (lane & 31);
            const int cc = cls < n ? cls : n - 1;
#pragma unroll
            for (int e = 0; e < 16; ++e) sa_old[i][j][e] = SA[(int64_t)fid[i][e] * n + cc];
        }

    for (int st = 0; st < n_stage; st += 4) {            // four stages per trip so the register sets are static
        // stage st: LDS buffer 0 holds it; set 0 is free, sets 1..3 hold stages st+1 .. st+3
        if (st + 4 < n_stage) fetch(ra0, rb0, st + 4);
        multiply(0);
        if (st + 1 < n_stage) stash(ra1, rb1, 1);        // buffer 1 was last read before the previous barrier
        __syncthreads();
        if (st + 1 >= n_stage) break;                    // uniform
        // stage st+1: buffer 1
        if (st + 5 < n_stage) fetch(ra1, rb1, st + 5);
        multiply(1);
        if (st + 2 < n_stage) stash(ra2, rb2, 0);
        __syncthreads();
        if (st + 2 >= n_stage) break;
        // stage st+2: buffer 0
        if (st + 6 < n_stage) fetch(ra2, rb2, st + 6);
        multiply(0);
        if (st + 3 < n_stage) stash(ra3, rb3, 1);
        __syncthreads();
        if (st + 3 >= n_stage) break;
        // stage st+3: buffer 1
        if (st + 7 < n_stage) fetch(ra3, rb3, st + 7);
        multiply(1);
        if (st + 4 < n_stage) stash(ra0, rb0, 0);
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int cls = n0 + (wn * WN + j) * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int slot = m0 + (wm * WM + i) * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (slot < n_live && cls < n) {
                    const float s = acc[i][j][e];
                    SA[(int64_t)fid[i][e] * n + cls] = sa_old[i][j][e] + weight * s;
                    if (sims_out) sims_out[(int64_t)slot * n + cls] = s;
                }
            }
        }
}

void launch_score_mfma(const _Float16* vhat, const _Float16* chat, int Cp, const int32_t* frame_ids,
                       const Counts* counts, int max_rows, int n, float weight, float* SA,
                       float* sims_out, hipStream_t st) {
    // operands are padded to kRowPad rows, so a 64x64 block tile never reads outside them
    dim3 grid((n + 63) / 64, (max_rows + 63) / 64);
    hipLaunchKernelGGL((k_score_mfma<1, 1>), grid, dim3(256), 0, st, vhat, chat, Cp, frame_ids, counts,
                       max_rows, n, weight, SA, sims_out);
}

// ---------------------------------------------------------------------------------------------
// Top-2 per tier and the exit rule.  One wavefront per live slot walks its SA row.
struct Top2 {
    float v1; int id1; float v2;
};

// The order is (larger value first, then smaller class id); id < 0 with value -inf marks "no entry".
// Accumulated similarities are finite, so -inf never is a real entry.  Everything below is written with
// selects: as nested branches the per-element update cost several times the memory traffic of the row.

// One more entry for a lane's running top-2.  A lane meets its classes in ascending id, so an equal value
// never displaces the best one (strict >).  `take` = false leaves the triple as it is.
__device__ __forceinline__ void top2_push(Top2& t, float v, int id, bool take = true) {
    const float x = take ? v : -__builtin_inff();
    const bool gt = x > t.v1;
    t.v2 = gt ? t.v1 : fmaxf(t.v2, x);
    t.id1 = gt ? id : t.id1;
    t.v1 = gt ? x : t.v1;
}

// Merge of another lane's (best, id, second) triple; the second of a triple never exceeds its best.
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

__global__ __launch_bounds__(256) void k_top2_decide(
    const float* __restrict__ SA, const int32_t* __restrict__ frame_ids,
    const Counts* __restrict__ counts, int max_rows, int n, const uint8_t* __restrict__ in_hot,
    int tiers, float tau, int32_t* __restrict__ decision, int32_t* __restrict__ label,
    float* __restrict__ top_val, int32_t* __restrict__ top_id, float* __restrict__ top_val_user,
    int32_t* __restrict__ top_id_user) {
    const int lane = threadIdx.x & 63;
    int slot = blockIdx.x * 4 + (threadIdx.x >> 6);
    int n_live = counts->n_live;
    int fid = slot < max_rows ? frame_ids[slot] : 0;      // fetched together with the live count, as in k_rownorm
    asm volatile("" : "+v"(fid), "+s"(n_live));
    if (n_live > max_rows) n_live = max_rows;
    const int n_waves = gridDim.x * 4;
    const float ninf = -__builtin_inff();
    const bool vec = (n & 3) == 0;
    for (; slot < n_live; slot += n_waves, fid = slot < n_live ? frame_ids[slot] : 0) {
        const float* row = SA + (int64_t)fid * n;
        Top2 hot = {ninf, -1, ninf}, all = {ninf, -1, ninf};
        if (vec) {
            // each lane takes 4 consecutive classes per access, four accesses in flight
            const f32x4* row4 = reinterpret_cast<const f32x4*>(row);
            const uint32_t* hot4 = reinterpret_cast<const uint32_t*>(in_hot);
            const int nq = n >> 2;
            for (int base = 0; base < nq; base += 256) {
                f32x4 x[4];
                uint32_t h[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = base + u * 64 + lane;
                    if (q < nq) { x[u] = row4[q]; h[u] = hot4[q]; }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = base + u * 64 + lane;
                    if (q < nq) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            top2_push(all, x[u][e], 4 * q + e);
                            top2_push(hot, x[u][e], 4 * q + e, ((h[u] >> (8 * e)) & 0xffu) != 0);
                        }
                    }
                }
            }
        } else {
            for (int j = lane; j < n; j += 64) {
                const float x = row[j];
                top2_push(all, x, j);
                top2_push(hot, x, j, in_hot[j] != 0);
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            float v1 = __shfl_xor(all.v1, off, 64); int id1 = __shfl_xor(all.id1, off, 64);
            float v2 = __shfl_xor(all.v2, off, 64);
            top2_merge(all, v1, id1, v2);
            v1 = __shfl_xor(hot.v1, off, 64); id1 = __shfl_xor(hot.id1, off, 64);
            v2 = __shfl_xor(hot.v2, off, 64);
            top2_merge(hot, v1, id1, v2);
        }
        if (lane == 0) {
            int d = 0, lab = -1;
            if (exit_rule(hot.v1, hot.v2, tau)) { d = 1; lab = hot.id1; }
            else if (tiers == 2 && exit_rule(all.v1, all.v2, tau)) { d = 2; lab = all.id1; }
            if (tiers != 2) { all.v1 = ninf; all.v2 = ninf; all.id1 = -1; }
            decision[slot] = d;
            label[slot] = lab;
            float* tv = top_val + (int64_t)slot * 4;
            tv[0] = hot.v1; tv[1] = hot.v2; tv[2] = all.v1; tv[3] = all.v2;
            top_id[slot * 2] = hot.id1; top_id[slot * 2 + 1] = all.id1;
            if (top_val_user) {
                float* u = top_val_user + (int64_t)slot * 4;
                u[0] = hot.v1; u[1] = hot.v2; u[2] = all.v1; u[3] = all.v2;
            }
            if (top_id_user) { top_id_user[slot * 2] = hot.id1; top_id_user[slot * 2 + 1] = all.id1; }
        }
    }
}

// Single-layer separability (Eq. 2): sep = (s_H - s_SH) / s_SH over one exit point's similarities,
// per tier.  A diagnostic, not on the decision path.  One wavefront per live slot.
// +inf where s_SH <= 0 < s_H, -inf where s_H <= 0 or the tier has fewer than two entries.
__global__ __launch_bounds__(256) void k_separability(const float* __restrict__ sims,
                                                      const Counts* __restrict__ counts, int max_rows, int n,
                                                      const uint8_t* __restrict__ in_hot,
                                                      float* __restrict__ sep_out) {
    const int lane = threadIdx.x & 63;
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int n_waves = gridDim.x * 4;
    const float ninf = -__builtin_inff();
    for (int slot = blockIdx.x * 4 + (threadIdx.x >> 6); slot < n_live; slot += n_waves) {
        const float* row = sims + (int64_t)slot * n;
        Top2 hot = {ninf, -1, ninf}, all = {ninf, -1, ninf};
        for (int j = lane; j < n; j += 64) {
            const float x = row[j];
            top2_push(all, x, j);
            top2_push(hot, x, j, in_hot[j] != 0);
        }
        for (int off = 32; off > 0; off >>= 1) {
            float v1 = __shfl_xor(all.v1, off, 64); int id1 = __shfl_xor(all.id1, off, 64);
            float v2 = __shfl_xor(all.v2, off, 64);
            top2_merge(all, v1, id1, v2);
            v1 = __shfl_xor(hot.v1, off, 64); id1 = __shfl_xor(hot.id1, off, 64);
            v2 = __shfl_xor(hot.v2, off, 64);
            top2_merge(hot, v1, id1, v2);
        }
        if (lane < 2) {
            const Top2 t = lane == 0 ? hot : all;
            float sep;
            if (!(t.v1 > 0.f) || t.v2 == ninf) sep = ninf;
            else if (!(t.v2 > 0.f)) sep = __builtin_inff();
            else sep = (t.v1 - t.v2) / t.v2;
            sep_out[slot * 2 + lane] = sep;
        }
    }
}

void launch_separability(const float* sims, const Counts* counts, int max_rows, int n, const uint8_t* in_hot,
                         float* sep_out, hipStream_t st) {
    int grid = (max_rows + 3) / 4;
    if (grid > 2048) grid = 2048;
    hipLaunchKernelGGL(k_separability, grid, dim3(256), 0, st, sims, counts, max_rows, n, in_hot, sep_out);
}

void launch_top2_decide(const float* SA, const int32_t* frame_ids, const Counts* counts, int max_rows,
                        int n, const uint8_t* in_hot, int tiers, float tau, int32_t* decision,
                        int32_t* label, float* top_val, int32_t* top_id, float* top_val_user,
                        int32_t* top_id_user, hipStream_t st) {
    int grid = (max_rows + 3) / 4;
    if (grid > 2048) grid = 2048;
    hipLaunchKernelGGL(k_top2_decide, grid, dim3(256), 0, st, SA, frame_ids, counts, max_rows, n, in_hot,
                       tiers, tau, decision, label, top_val, top_id, top_val_user, top_id_user);
}

}  // namespace smtm
