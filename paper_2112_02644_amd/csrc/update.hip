// Memory update between batches (arXiv 2112.02644, Sec. 6): frequency and time-stamp tables
// (Sec. 6.1), replacement score (Eq. 5), adaptive fast-memory size (Eq. 6), adaptive centres
// (Eq. 7).  Tables, scores, order and size are exact integer work; only the centres are
// floating point.  All of it is a few thousand entries: latency-bound, one or a few blocks.
#include "internal.h"

namespace smtm {

typedef unsigned __int128 u128;

// Frequency / time-stamp tables for a whole batch, equal to taking the frames one by one:
// FT_j += (appearances of j);  TS_j = (frames after j's last appearance) if j appeared,
// else TS_j + batch.  Both saturate at 2^32 - 1.  Single block.
__global__ __launch_bounds__(1024) void k_tables_update(const int32_t* __restrict__ label, int batch,
                                                        int n, uint32_t* __restrict__ FT,
                                                        uint32_t* __restrict__ TS,
                                                        uint32_t* __restrict__ cls_cnt,
                                                        int32_t* __restrict__ cls_last) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) { cls_cnt[i] = 0; cls_last[i] = -1; }
    __syncthreads();
    for (int b = threadIdx.x; b < batch; b += blockDim.x) {
        const int j = label[b];
        if (j >= 0 && j < n) {
            atomicAdd(&cls_cnt[j], 1u);
            atomicMax(&cls_last[j], b);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const uint64_t ft = (uint64_t)FT[i] + cls_cnt[i];
        FT[i] = ft > 0xffffffffull ? 0xffffffffu : (uint32_t)ft;
        uint64_t ts;
        if (cls_last[i] >= 0) ts = (uint64_t)(batch - 1 - cls_last[i]);
        else ts = (uint64_t)TS[i] + (uint64_t)batch;
        TS[i] = ts > 0xffffffffull ? 0xffffffffu : (uint32_t)ts;
    }
}

void launch_tables_update(const int32_t* label, int batch, int n, uint32_t* FT, uint32_t* TS,
                          uint32_t* cls_cnt, int32_t* cls_last, hipStream_t st) {
    hipLaunchKernelGGL(k_tables_update, dim3(1), dim3(1024), 0, st, label, batch, n, FT, TS, cls_cnt,
                       cls_last);
}

// Adaptive centres (Eq. 7) for one exit point.  Taking the frames of class j one by one gives
// the running mean (m*SC + sum of their SV) / (m + count); the sum is taken in ascending frame
// order so the result does not depend on scheduling.  One block per class that appeared; the
// block also refreshes 1/|SC_j| and the unit fp16 copy.
__global__ __launch_bounds__(256) void k_centres_update(
    float* __restrict__ centres, uint32_t* __restrict__ mcount, float* __restrict__ cinv,
    _Float16* __restrict__ chat, int Cp, const float* __restrict__ sv, int C, int n, int exit_index,
    const int32_t* __restrict__ label, const int32_t* __restrict__ stop_layer, int batch,
    const uint32_t* __restrict__ cls_cnt) {
    __shared__ float red[4];
    __shared__ int s_cnt;
    const int j = blockIdx.x;
    if (j >= n || cls_cnt[j] == 0) return;               // uniform over the block
    const int tid = threadIdx.x;
    float* sc = centres + (int64_t)j * C;
    const float m = (float)mcount[j];
    // count the frames that update this exit point (label == j and stopped at or after it)
    int cnt = 0;
    float ss = 0.f;
    for (int c0 = 0; c0 < C; c0 += 256) {                // uniform trip count
        const int c = c0 + tid;
        float sum = 0.f;
        cnt = 0;
        for (int b = 0; b < batch; ++b) {
            if (label[b] == j && stop_layer[b] > exit_index) {
                ++cnt;
                if (c < C) sum += sv[(int64_t)b * C + c];
            }
        }
        if (c < C && cnt > 0) {
            const float x = (sc[c] * m + sum) / (m + (float)cnt);
            sc[c] = x;
            ss += x * x;
        } else if (c < C) {
            const float x = sc[c];
            ss += x * x;
        }
    }
    if (tid == 0) s_cnt = cnt;
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (s_cnt == 0) return;                              // uniform: nothing changed at this exit point
    const float nrm2 = (red[0] + red[1]) + (red[2] + red[3]);
    float inv = 0.f;
    if (nrm2 > 0.f && nrm2 < __builtin_inff()) inv = 1.0f / sqrtf(nrm2);
    if (tid == 0) {
        cinv[j] = inv;
        const uint64_t mm = (uint64_t)mcount[j] + (uint64_t)s_cnt;
        mcount[j] = mm > 0xffffffffull ? 0xffffffffu : (uint32_t)mm;
    }
    for (int c = tid; c < Cp; c += 256) {
        float x = 0.f;
        if (c < C && inv != 0.f) x = sc[c] * inv;       // sc[c] was written by this same thread (c % 256 == tid)
        chat[(int64_t)j * Cp + c] = (_Float16)x;
    }
}

void launch_centres_update(float* centres, uint32_t* mcount, float* cinv, _Float16* chat, int Cp,
                           const float* sv, int C, int n, int exit_index, const int32_t* label,
                           const int32_t* stop_layer, int batch, const uint32_t* cls_cnt,
                           hipStream_t st) {
    hipLaunchKernelGGL(k_centres_update, dim3(n), dim3(256), 0, st, centres, mcount, cinv, chat, Cp, sv, C,
                       n, exit_index, label, stop_layer, batch, cls_cnt);
}

// Replacement policy and adaptive size.  Single block of 1024 threads.
//   score_i = FT_i * 4^(15 - min(floor(TS_i / W), 15))       (Eq. 5 scaled by 4^15, exact)
//   rank_i  = number of classes ahead of i in (score desc, id asc) order
//   k       = 1 + number of ranks whose inclusive prefix sum is still below CL * total
//             (the prefix share is non-decreasing in the rank), clamped to [hot_min, hot_max]
__device__ __forceinline__ uint64_t score_of(uint32_t ft, uint32_t ts, uint32_t W) {
    uint32_t q = ts / W;
    if (q > 15u) q = 15u;
    return (uint64_t)ft << (2u * (15u - q));
}

__global__ __launch_bounds__(1024) void k_policy(const uint32_t* __restrict__ FT,
                                                 const uint32_t* __restrict__ TS, int n, uint32_t W,
                                                 uint32_t cl_num, uint32_t cl_den, int hot_min,
                                                 int hot_max, uint64_t* __restrict__ score,
                                                 int32_t* __restrict__ order,
                                                 int32_t* __restrict__ hot_ids,
                                                 uint8_t* __restrict__ in_hot,
                                                 Counts* __restrict__ counts) {
    __shared__ uint64_t red_lo[1024], red_hi[1024];
    __shared__ int red_cnt[1024];
    const int tid = threadIdx.x;
    u128 part = 0;
    for (int i = tid; i < n; i += 1024) {
        const uint64_t s = score_of(FT[i], TS[i], W);
        score[i] = s;
        part += s;
    }
    red_lo[tid] = (uint64_t)part; red_hi[tid] = (uint64_t)(part >> 64);
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if (tid < off) {
            u128 a = ((u128)red_hi[tid] << 64) | red_lo[tid];
            u128 b = ((u128)red_hi[tid + off] << 64) | red_lo[tid + off];
            a += b;
            red_lo[tid] = (uint64_t)a; red_hi[tid] = (uint64_t)(a >> 64);
        }
        __syncthreads();
    }
    const u128 total = ((u128)red_hi[0] << 64) | red_lo[0];
    if (total == 0) return;                              // no history: the fast memory stays as it is
    const u128 need = total * cl_num;                    // prefix * cl_den >= total * cl_num
    int below = 0;
    for (int i = tid; i < n; i += 1024) {
        const uint64_t si = score[i];
        int rank = 0;
        u128 prefix = si;                                // inclusive prefix sum at i's rank
        for (int j = 0; j < n; ++j) {
            const uint64_t sj = score[j];
            if (sj > si || (sj == si && j < i)) { ++rank; prefix += sj; }
        }
        order[rank] = i;
        if (prefix * cl_den < need) ++below;
    }
    red_cnt[tid] = below;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if (tid < off) red_cnt[tid] += red_cnt[tid + off];
        __syncthreads();
    }
    int k = red_cnt[0] + 1;
    if (k < hot_min) k = hot_min;
    if (k > hot_max) k = hot_max;
    for (int i = tid; i < n; i += 1024) in_hot[i] = 0;
    __syncthreads();                                     // order[] and in_hot[] writes of this block are visible
    for (int r = tid; r < k; r += 1024) {
        const int id = order[r];
        hot_ids[r] = id;
        in_hot[id] = 1;
    }
    if (tid == 0) counts->hot_k = k;
}

void launch_policy(const uint32_t* FT, const uint32_t* TS, int n, uint32_t W, uint32_t cl_num,
                   uint32_t cl_den, int hot_min, int hot_max, uint64_t* score, int32_t* order,
                   int32_t* hot_ids, uint8_t* in_hot, Counts* counts, hipStream_t st) {
    hipLaunchKernelGGL(k_policy, dim3(1), dim3(1024), 0, st, FT, TS, n, W, cl_num, cl_den, hot_min,
                       hot_max, score, order, hot_ids, in_hot, counts);
}

}  // namespace smtm
