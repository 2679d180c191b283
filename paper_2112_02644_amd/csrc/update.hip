// Memory update between batches (arXiv 2112.02644, Sec. 6): frequency and time-stamp tables
// (Sec. 6.1), replacement score (Eq. 5), adaptive fast-memory size (Eq. 6), adaptive centres
// (Eq. 7).  Tables, scores, order and size are exact integer work; only the centres are
// floating point.  All of it is a few thousand entries: latency-bound, so the work is spread
// over many short lanes rather than a few long loops.
#include <mutex>

#include "internal.h"

namespace smtm {

typedef unsigned __int128 u128;
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint64_t score_of(uint32_t ft, uint32_t ts, uint32_t W) {
    // Eq. 5 scaled by 4^15: FT * 4^(15 - min(floor(TS / W), 15)), exact in 64 bits
    uint32_t q = ts / W;
    if (q > 15u) q = 15u;
    return (uint64_t)ft << (2u * (15u - q));
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t x, int off) {
    uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    lo = __shfl_xor(lo, off, 64);
    hi = __shfl_xor(hi, off, 64);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ u128 shfl_xor_u128(u128 x, int off) {
    return ((u128)shfl_xor_u64((uint64_t)(x >> 64), off) << 64) | shfl_xor_u64((uint64_t)x, off);
}

// Frequency / time-stamp tables for a whole batch, equal to taking the frames one by one:
// FT_j += (appearances of j);  TS_j = (frames after j's last appearance) if j appeared,
// else TS_j + batch.  Both saturate at 2^32 - 1.  With `inplace` the forgetting of Sec. 6.1 is applied
// to the counts as the frames go by instead of at scoring time.  Also leaves every class's score and the
// 128-bit total of the scores (total[0] low, total[1] high) and clears the policy counter.
// Single block of 1024 threads.
constexpr int kLdsClasses = 4096;
constexpr int kLabelTile = 4096;

__global__ __launch_bounds__(1024) void k_tables_update(const int32_t* __restrict__ label, int batch,
                                                        int n, uint32_t W, uint32_t* __restrict__ FT,
                                                        uint32_t* __restrict__ TS,
                                                        uint32_t* __restrict__ cls_cnt,
                                                        int32_t* __restrict__ cls_last,
                                                        uint64_t* __restrict__ score,
                                                        uint64_t* __restrict__ total,
                                                        int32_t* __restrict__ below, int inplace) {
    __shared__ uint64_t red_lo[16], red_hi[16];
    __shared__ uint32_t l_cnt[kLdsClasses];
    __shared__ int32_t l_last[kLdsClasses];
    __shared__ int32_t l_lab[kLabelTile];
    const int tid = threadIdx.x;
    const bool in_lds = n <= kLdsClasses;                // histogram in LDS when the classes fit, else in global memory
    for (int i = tid; i < n; i += 1024) {
        if (in_lds) { l_cnt[i] = 0; l_last[i] = -1; } else { cls_cnt[i] = 0; cls_last[i] = -1; }
    }
    __syncthreads();
    for (int b = tid; b < batch; b += 1024) {
        const int j = label[b];
        if (j >= 0 && j < n) {
            if (in_lds) { atomicAdd(&l_cnt[j], 1u); atomicMax(&l_last[j], b); }
            else { atomicAdd(&cls_cnt[j], 1u); atomicMax(&cls_last[j], b); }
        }
    }
    __syncthreads();
    u128 part = 0;
    if (inplace) {
        // Forgetting applied to the frequency table itself (Sec. 6.1): thread = class, the batch's
        // labels are walked in order; every W-th consecutive frame without the class quarters its count.
        for (int c0 = 0; c0 < n; c0 += 1024) {           // uniform trip counts: the label tiles are shared
            const int i = c0 + tid;
            const bool valid = i < n;
            uint32_t ft = valid ? FT[i] : 0u, ts = valid ? TS[i] : 0u;
            uint32_t left = W - ts % W;                  // frames until TS reaches the next multiple of W
            for (int b0 = 0; b0 < batch; b0 += kLabelTile) {
                const int len = batch - b0 < kLabelTile ? batch - b0 : kLabelTile;
                __syncthreads();
                for (int b = tid; b < len; b += 1024) l_lab[b] = label[b0 + b];
                __syncthreads();
                if (valid) {
                    for (int b = 0; b < len; ++b) {
                        if (l_lab[b] == i) {
                            ts = 0u; left = W;
                            if (ft != 0xffffffffu) ++ft;
                        } else if (ts != 0xffffffffu) {
                            ++ts;
                            if (--left == 0u) { ft >>= 2; left = W; }
                        }
                    }
                }
            }
            if (valid) {
                if (in_lds) cls_cnt[i] = l_cnt[i];       // the centre update reads the counts
                FT[i] = ft; TS[i] = ts;
                score[i] = (uint64_t)ft;                 // the decay is already in the count
                part += ft;
            }
        }
    } else
    for (int i = tid; i < n; i += 1024) {
        const uint32_t cnt_i = in_lds ? l_cnt[i] : cls_cnt[i];
        const int32_t last_i = in_lds ? l_last[i] : cls_last[i];
        if (in_lds) cls_cnt[i] = cnt_i;                  // the centre update reads the counts
        uint64_t ft = (uint64_t)FT[i] + cnt_i;
        if (ft > 0xffffffffull) ft = 0xffffffffull;
        uint64_t ts;
        if (last_i >= 0) ts = (uint64_t)(batch - 1 - last_i);
        else ts = (uint64_t)TS[i] + (uint64_t)batch;
        if (ts > 0xffffffffull) ts = 0xffffffffull;
        FT[i] = (uint32_t)ft;
        TS[i] = (uint32_t)ts;
        const uint64_t s = score_of((uint32_t)ft, (uint32_t)ts, W);
        score[i] = s;
        part += s;
    }
    for (int off = 32; off > 0; off >>= 1) part += shfl_xor_u128(part, off);
    if ((tid & 63) == 0) { red_lo[tid >> 6] = (uint64_t)part; red_hi[tid >> 6] = (uint64_t)(part >> 64); }
    __syncthreads();
    if (tid == 0) {
        u128 t = 0;
        for (int w = 0; w < 16; ++w) t += ((u128)red_hi[w] << 64) | red_lo[w];
        total[0] = (uint64_t)t; total[1] = (uint64_t)(t >> 64);
        *below = 0;
    }
}

void launch_tables_update(const int32_t* label, int batch, int n, uint32_t W, uint32_t* FT, uint32_t* TS,
                          uint32_t* cls_cnt, int32_t* cls_last, uint64_t* score, uint64_t* total,
                          int32_t* below, int inplace, hipStream_t st) {
    hipLaunchKernelGGL(k_tables_update, dim3(1), dim3(1024), 0, st, label, batch, n, W, FT, TS, cls_cnt,
                       cls_last, score, total, below, inplace);
}

// Appearances of every class in a batch of labels (nothing else is touched).  Single block.
__global__ __launch_bounds__(1024) void k_class_count(const int32_t* __restrict__ label, int batch, int n,
                                                      uint32_t* __restrict__ cls_cnt) {
    for (int i = threadIdx.x; i < n; i += 1024) cls_cnt[i] = 0;
    __syncthreads();
    for (int b = threadIdx.x; b < batch; b += 1024) {
        const int j = label[b];
        if (j >= 0 && j < n) atomicAdd(&cls_cnt[j], 1u);
    }
}

void launch_class_count(const int32_t* label, int batch, int n, uint32_t* cls_cnt, hipStream_t st) {
    hipLaunchKernelGGL(k_class_count, dim3(1), dim3(1024), 0, st, label, batch, n, cls_cnt);
}

// Adaptive centres (Eq. 7), all exit points in one launch: block (j, l0) handles class j at
// exit point l0.  Taking the frames of class j one by one gives the running mean
// (m*SC + sum of their SV) / (m + count); the sum is taken in ascending frame order, so the
// result does not depend on scheduling.  The block lists the frames that update it (label == j
// and stopped at or after this exit point) with a ballot/prefix pass over the labels, then
// each thread adds up its channels over that list.  It also refreshes 1/|SC_j| and the unit
// fp16 copy of the row.
constexpr int kListCap = 4096;

// A frame's saved semantic vectors exist only for the exit points it was live at: one that the library
// released at exit point r has them for 1..r, one that ran on has them for the exit points encoded in
// this batch (1..enc_upto).  A larger stop_layer is cut down to that.
__device__ __forceinline__ int usable_stop(int stop, int released_at, int enc_upto) {
    const int have = released_at > 0 ? released_at : enc_upto;
    return stop < have ? stop : have;
}

__device__ __forceinline__ void centres_block(const CentreTables& tabs, const int32_t* __restrict__ label,
                                              const int32_t* __restrict__ stop_layer, int batch,
                                              const uint32_t* __restrict__ cls_cnt, int j, int l0) {
    const int32_t* __restrict__ res_layer = tabs.res_layer;
    const int enc_upto = tabs.enc_upto;
    __shared__ int list[kListCap];
    __shared__ int w_cnt[4];
    __shared__ float red[4];
    __shared__ float part[256];
    if (cls_cnt[j] == 0) return;                         // uniform over the block
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int C = tabs.C[l0], Cp = tabs.Cp[l0];
    float* sc = tabs.centres[l0] + (int64_t)j * C;
    const float* sv = tabs.sv[l0];
    const int32_t* __restrict__ slot_of = tabs.slot_of[l0];

    // frames of this class that reached this exit point, ascending.  A thread looks at four consecutive
    // frames per pass (one 16-byte load from each array when they are aligned), so a batch of 1024 is one
    // pass; its hits go behind those of the lower lanes and wavefronts, which keeps the list in frame order.
    int cnt = 0;
    bool overflow = false;
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(label) | reinterpret_cast<uintptr_t>(stop_layer) |
                          reinterpret_cast<uintptr_t>(res_layer)) & 15u) == 0;
    for (int b0 = 0; b0 < batch; b0 += 1024) {           // uniform trip count
        const int b = b0 + 4 * tid;
        int lab[4] = {-1, -1, -1, -1}, stp[4] = {0, 0, 0, 0};
        if (vec_ok && b + 3 < batch) {
            const i32x4 lv = *reinterpret_cast<const i32x4*>(label + b);
            const i32x4 sv4 = *reinterpret_cast<const i32x4*>(stop_layer + b);
            const i32x4 rl4 = *reinterpret_cast<const i32x4*>(res_layer + b);
#pragma unroll
            for (int k = 0; k < 4; ++k) { lab[k] = lv[k]; stp[k] = usable_stop(sv4[k], rl4[k], enc_upto); }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (b + k < batch) { lab[k] = label[b + k]; stp[k] = usable_stop(stop_layer[b + k], res_layer[b + k], enc_upto); }
        }
        bool hit[4];
        int pre = 0, tot_w = 0, own = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            hit[k] = lab[k] == j && stp[k] > l0;
            const unsigned long long m = __ballot(hit[k]);
            pre += __popcll(m & ((1ull << lane) - 1ull));
            tot_w += __popcll(m);
        }
        if (lane == 0) w_cnt[wave] = tot_w;
        __syncthreads();
        int off = 0, tot = 0;
        for (int w = 0; w < 4; ++w) { if (w < wave) off += w_cnt[w]; tot += w_cnt[w]; }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (hit[k]) {
                const int pos = cnt + off + pre + own;
                if (pos < kListCap) list[pos] = slot_of[b + k];      // where the frame's vector of this exit point is
                ++own;
            }
        }
        cnt += tot;
        __syncthreads();
    }
    if (cnt == 0) return;                                // uniform: nothing to do at this exit point
    overflow = cnt > kListCap;
    const float m_old = (float)tabs.mcount[l0][j];
    float ss = 0.f;
    // thread = channel (256 at a time, coalesced rows), frames of the list in ascending order, up to 32
    // rows in flight.  Narrow layers (C <= 128) put 256 / Cw threads on each channel (Cw = C rounded
    // up to a power of two): thread (g, c) adds the frames g, g + G, ... of the list and the G partial
    // sums meet in LDS in the order of g, so the result does not depend on the launch.
    int Cw = 256, G = 1;
    if (C <= 128 && !overflow) {
        Cw = 1;
        while (Cw < C) Cw <<= 1;
        G = 256 / Cw;
    }
    if (G > 1) {
        const int g = tid / Cw, c = tid - g * Cw;
        float sum = 0.f;
        if (c < C) {
            int i = g;
            for (; i + 7 * G < cnt; i += 8 * G) {
                float a[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) a[u] = sv[(int64_t)list[i + u * G] * Cp + c];
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += a[u];
            }
            if (i < cnt) {                               // the rest (fewer than 8 of this group) in one batch
                float a[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int k = i + u * G;
                    a[u] = sv[(int64_t)list[k < cnt ? k : i] * Cp + c];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += i + u * G < cnt ? a[u] : 0.f;
            }
        }
        part[tid] = sum;
        __syncthreads();
        if (g == 0 && c < C) {
            float tot = part[c];
            for (int k = 1; k < G; ++k) tot += part[k * Cw + c];
            const float x = (sc[c] * m_old + tot) / (m_old + (float)cnt);
            sc[c] = x;
            ss += x * x;
        }
    } else {
        for (int c = tid; c < C; c += 256) {
            float sum = 0.f;
            if (!overflow) {
                int i = 0;
                for (; i + 32 <= cnt; i += 32) {
                    float a[32];
#pragma unroll
                    for (int u = 0; u < 32; ++u) a[u] = sv[(int64_t)list[i + u] * Cp + c];
#pragma unroll
                    for (int u = 0; u < 32; ++u) sum += a[u];
                }
                // the rest (fewer than 32 frames) in one batch: indices past the end are clamped and their
                // values dropped, so the loads need no branch and the order of the additions stays the list's
                if (cnt - i > 8) {
                    float a[32];
#pragma unroll
                    for (int u = 0; u < 32; ++u) a[u] = sv[(int64_t)list[i + u < cnt ? i + u : i] * Cp + c];
#pragma unroll
                    for (int u = 0; u < 32; ++u) sum += i + u < cnt ? a[u] : 0.f;
                } else if (cnt > i) {
                    float a[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) a[u] = sv[(int64_t)list[i + u < cnt ? i + u : i] * Cp + c];
#pragma unroll
                    for (int u = 0; u < 8; ++u) sum += i + u < cnt ? a[u] : 0.f;
                }
            } else {                                     // more frames of one class than the list holds
                for (int b = 0; b < batch; ++b)
                    if (label[b] == j && usable_stop(stop_layer[b], res_layer[b], enc_upto) > l0) sum += sv[(int64_t)slot_of[b] * Cp + c];
            }
            const float x = (sc[c] * m_old + sum) / (m_old + (float)cnt);
            sc[c] = x;
            ss += x * x;
        }
    }
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    const float nrm2 = (red[0] + red[1]) + (red[2] + red[3]);
    float inv = 0.f;
    if (nrm2 > 0.f && nrm2 < __builtin_inff()) inv = 1.0f / sqrtf(nrm2);
    if (tid == 0) {
        tabs.cinv[l0][j] = inv;
        const uint64_t mm = (uint64_t)tabs.mcount[l0][j] + (uint64_t)cnt;
        tabs.mcount[l0][j] = mm > 0xffffffffull ? 0xffffffffu : (uint32_t)mm;
    }
    _Float16* ch = tabs.chat[l0];
    for (int c = tid; c < Cp; c += 256) {
        float x = 0.f;
        if (c < C && inv != 0.f) x = sc[c] * inv;        // sc[c] was written by this same thread
        ch[chat_index(j, c, Cp)] = (_Float16)x;
    }
}

__global__ __launch_bounds__(256) void k_centres_update(CentreTables tabs, int n, const int32_t* __restrict__ label,
                                                        const int32_t* __restrict__ stop_layer, int batch,
                                                        const uint32_t* __restrict__ cls_cnt) {
    centres_block(tabs, label, stop_layer, batch, cls_cnt, blockIdx.x, blockIdx.y);
}

void launch_centres_update(const CentreTables& tabs, int n_exits, int n, const int32_t* label,
                           const int32_t* stop_layer, int batch, const uint32_t* cls_cnt, hipStream_t st) {
    hipLaunchKernelGGL(k_centres_update, dim3(n, n_exits), dim3(256), 0, st, tabs, n, label, stop_layer,
                       batch, cls_cnt);
}

// Replacement policy and adaptive size (Eq. 5, Eq. 6).
//   rank_i  = number of classes ahead of i in (score desc, id asc) order
//   prefix_i = sum of the scores of the classes up to and including i in that order
//   k       = 1 + number of classes whose prefix is still below CL * total
//             (the prefix share is non-decreasing along the order), clamped to [hot_min, hot_max]
// rank_block: 16 lanes per class split the scan over all classes and combine with shuffles.
// The ranks only need the scores, the centres only the class counts: both come from
// k_tables_update, so the two share one launch (k_centres_and_rank) and run side by side.
constexpr int kRankTile = 2048;            // scores staged per pass (16 KB of LDS)

__device__ __forceinline__ void rank_block(const uint64_t* __restrict__ score,
                                           const uint64_t* __restrict__ total, int n,
                                           uint32_t cl_num, uint32_t cl_den,
                                           int32_t* __restrict__ order,
                                           int32_t* __restrict__ below, int block) {
    __shared__ uint64_t tile[kRankTile];
    const int tid = threadIdx.x, sub = tid & 15;
    const int i = block * 16 + (tid >> 4);
    const bool valid = i < n;
    const uint64_t si = valid ? score[i] : 0;            // issued before the total is needed
    const u128 tot = ((u128)total[1] << 64) | total[0];
    if (tot == 0) return;                                // no history: nothing changes (uniform)
    int rank = 0;
    u128 prefix = 0;
    for (int j0 = 0; j0 < n; j0 += kRankTile) {          // uniform trip count
        const int len = n - j0 < kRankTile ? n - j0 : kRankTile;
        for (int j = tid; j < len; j += 256) tile[j] = score[j0 + j];
        __syncthreads();
        if (valid) {
#pragma unroll 4
            for (int j = sub; j < len; j += 16) {
                const uint64_t sj = tile[j];
                const int jj = j0 + j;
                if (sj > si || (sj == si && jj < i)) { ++rank; prefix += sj; }
            }
        }
        __syncthreads();
    }
    for (int off = 8; off > 0; off >>= 1) {
        rank += __shfl_xor(rank, off, 64);
        prefix += shfl_xor_u128(prefix, off);
    }
    if (valid && sub == 0) {
        prefix += si;
        order[rank] = i;
        if (prefix * cl_den < tot * cl_num) atomicAdd(below, 1);
    }
}

__global__ __launch_bounds__(256) void k_centres_and_rank(CentreTables tabs, int n_exits, int n,
                                                          const int32_t* __restrict__ label,
                                                          const int32_t* __restrict__ stop_layer, int batch,
                                                          const uint32_t* __restrict__ cls_cnt,
                                                          const uint64_t* __restrict__ score,
                                                          const uint64_t* __restrict__ total,
                                                          uint32_t cl_num, uint32_t cl_den,
                                                          int32_t* __restrict__ order,
                                                          int32_t* __restrict__ below) {
    const int n_rank = (n + 15) / 16;                    // the rank blocks come first: all of them have work
    const int b = blockIdx.x;
    if (b < n_rank) {
        rank_block(score, total, n, cl_num, cl_den, order, below, b);
    } else {
        const int r = b - n_rank;
        centres_block(tabs, label, stop_layer, batch, cls_cnt, r % n, r / n);
    }
}

__global__ __launch_bounds__(1024) void k_policy_finish(const uint64_t* __restrict__ total, int n,
                                                        int hot_min, int hot_max,
                                                        const int32_t* __restrict__ order,
                                                        const int32_t* __restrict__ below,
                                                        int32_t* __restrict__ hot_ids,
                                                        uint8_t* __restrict__ in_hot,
                                                        Counts* __restrict__ counts) {
    if ((total[0] | total[1]) == 0) return;              // no history: the fast memory stays as it is
    const int tid = threadIdx.x;
    int k = *below + 1;
    if (k < hot_min) k = hot_min;
    if (k > hot_max) k = hot_max;
    for (int i = tid; i < n; i += 1024) in_hot[i] = 0;
    __syncthreads();
    for (int r = tid; r < k; r += 1024) {
        const int id = order[r];
        hot_ids[r] = id;
        in_hot[id] = 1;
    }
    if (tid == 0) counts->hot_k = k;
}

void launch_centres_and_policy(const CentreTables& tabs, int n_exits, int n, const int32_t* label,
                               const int32_t* stop_layer, int batch, const uint32_t* cls_cnt,
                               const uint64_t* score, const uint64_t* total, uint32_t cl_num, uint32_t cl_den,
                               int hot_min, int hot_max, int32_t* order, int32_t* below, int32_t* hot_ids,
                               uint8_t* in_hot, Counts* counts, hipStream_t st) {
    const int blocks = (n + 15) / 16 + n * n_exits;
    hipLaunchKernelGGL(k_centres_and_rank, dim3(blocks), dim3(256), 0, st, tabs, n_exits, n, label, stop_layer,
                       batch, cls_cnt, score, total, cl_num, cl_den, order, below);
    hipLaunchKernelGGL(k_policy_finish, dim3(1), dim3(1024), 0, st, total, n, hot_min, hot_max, order, below,
                       hot_ids, in_hot, counts);
}

// ---------------------------------------------------------------------------------------------
// Scratch of the memory update for callers that cannot allocate: one file-scope device array per
// GPU, laid out for up to kStaticMaxClasses classes.  The array's name is only a host-side handle;
// its device address is looked up once per GPU and that address is what kernels are given.
constexpr size_t kStaticAlign = 256;
constexpr size_t static_round(size_t x) { return (x + kStaticAlign - 1) / kStaticAlign * kStaticAlign; }
constexpr size_t kStaticOffCnt = 0;                                                        // uint32 [n]
constexpr size_t kStaticOffLast = kStaticOffCnt + static_round(4 * (size_t)kStaticMaxClasses);   // int32 [n]
constexpr size_t kStaticOffScore = kStaticOffLast + static_round(4 * (size_t)kStaticMaxClasses); // uint64 [n]
constexpr size_t kStaticOffOrder = kStaticOffScore + static_round(8 * (size_t)kStaticMaxClasses);// int32 [n]
constexpr size_t kStaticOffTotal = kStaticOffOrder + static_round(4 * (size_t)kStaticMaxClasses);// uint64 [2]
constexpr size_t kStaticOffBelow = kStaticOffTotal + kStaticAlign;                               // int32 [1]
constexpr size_t kStaticBytes = kStaticOffBelow + kStaticAlign;

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once known

hipError_t update_static_scratch(int device, UpdateScratch* out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    unsigned char* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[device]) {
            // the caller has made `device` current: the symbol is resolved for that GPU's copy of the array
            void* p = nullptr;
            const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[device] = static_cast<unsigned char*>(p);
        }
        base = g_scratch_ptr[device];
    }
    out->cls_cnt = reinterpret_cast<uint32_t*>(base + kStaticOffCnt);
    out->cls_last = reinterpret_cast<int32_t*>(base + kStaticOffLast);
    out->score = reinterpret_cast<uint64_t*>(base + kStaticOffScore);
    out->order = reinterpret_cast<int32_t*>(base + kStaticOffOrder);
    out->total = reinterpret_cast<uint64_t*>(base + kStaticOffTotal);
    out->below = reinterpret_cast<int32_t*>(base + kStaticOffBelow);
    return hipSuccess;
}

}  // namespace smtm
