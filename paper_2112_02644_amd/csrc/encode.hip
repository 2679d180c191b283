// Encode: semantic vector = global average pooling of each channel's H x W map
// (arXiv 2112.02644, Sec. 4.1).  The feature map is read exactly once, in place, with the
// widest loads its shape allows; sums are kept in fp32.
//
// Two streaming paths:
//   direct  a group of g lanes (g = 1..64, a power of two) owns one channel and walks it with
//           VB-byte loads, up to UNR loads in flight per lane; 64/g channels per wavefront.
//           Used when a channel's H*W*elem bytes are a multiple of VB.
//   pair    when a channel is a multiple of 8 but not of 16 bytes (14x14 fp16 = 392 B), two
//           neighbouring channels together are a multiple of 16: a lane group walks the pair
//           with 16-byte loads and splits the one chunk that straddles the two channels.
//   lds     for short, oddly sized channels (e.g. 7x7 fp16 = 98 B): a wavefront streams 64
//           consecutive channels (one contiguous piece of the frame) with 16-byte loads into
//           its own LDS region, then lane c adds up channel c from LDS.
// Work is taken in a grid-stride loop bounded by the live count read on the device.
#include <stdio.h>

#include "internal.h"

namespace smtm {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float sum_halves(uint32_t w) {
    half2_t h = __builtin_bit_cast(half2_t, w);
    return (float)h.x + (float)h.y;
}

template <typename T, int VB> struct Chunk;

template <> struct Chunk<_Float16, 16> {
    typedef u32x4 V;
    static __device__ __forceinline__ float sum(V v) {
        return (sum_halves(v.x) + sum_halves(v.y)) + (sum_halves(v.z) + sum_halves(v.w));
    }
};
template <typename T> struct Halves;          // sums of the lower and upper 8 bytes of a 16-byte chunk
template <> struct Halves<_Float16> {
    static __device__ __forceinline__ float lo(u32x4 v) { return sum_halves(v.x) + sum_halves(v.y); }
    static __device__ __forceinline__ float hi(u32x4 v) { return sum_halves(v.z) + sum_halves(v.w); }
};
template <> struct Halves<float> {
    // the whole vector is reinterpreted at once (a bit cast of a single vector element is not used here)
    static __device__ __forceinline__ float lo(u32x4 v) { const f32x4 f = __builtin_bit_cast(f32x4, v); return f.x + f.y; }
    static __device__ __forceinline__ float hi(u32x4 v) { const f32x4 f = __builtin_bit_cast(f32x4, v); return f.z + f.w; }
};

template <> struct Chunk<_Float16, 8> {
    typedef u32x2 V;
    static __device__ __forceinline__ float sum(V v) { return sum_halves(v.x) + sum_halves(v.y); }
};
template <> struct Chunk<_Float16, 4> {
    typedef uint32_t V;
    static __device__ __forceinline__ float sum(V v) { return sum_halves(v); }
};
template <> struct Chunk<_Float16, 2> {
    typedef _Float16 V;
    static __device__ __forceinline__ float sum(V v) { return (float)v; }
};
template <> struct Chunk<float, 16> {
    typedef f32x4 V;
    static __device__ __forceinline__ float sum(V v) { return (v.x + v.y) + (v.z + v.w); }
};
template <> struct Chunk<float, 8> {
    typedef f32x2 V;
    static __device__ __forceinline__ float sum(V v) { return v.x + v.y; }
};
template <> struct Chunk<float, 4> {
    typedef float V;
    static __device__ __forceinline__ float sum(V v) { return v; }
};

// GL >= 0 fixes the lanes per channel (2^GL) at compile time, which the 16-byte path uses: the
// load offsets and the reduction tree become constants.  GL < 0 takes it from the argument.
template <typename T, int VB, int UNR, int GL>
__global__ __launch_bounds__(256) void k_encode_direct(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    float* __restrict__ sv, float* __restrict__ sv_out, int C, int HW, int g_log2_arg) {
    typedef typename Chunk<T, VB>::V V;
    const int g_log2 = GL >= 0 ? GL : g_log2_arg;
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int n_waves = gridDim.x * (blockDim.x >> 6);
    const int g = 1 << g_log2;
    const int sub = lane & (g - 1);
    const int grp = lane >> g_log2;
    const int cpw = 64 >> g_log2;                       // channels per wavefront task
    const int tpf = (C + cpw - 1) / cpw;                // tasks per frame
    const int nv = (int)((int64_t)HW * sizeof(T) / VB); // chunks per channel
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int64_t total = (int64_t)n_live * tpf;

    for (int64_t t = wave; t < total; t += n_waves) {
        const int slot = (int)(t / tpf);
        const int c = (int)(t - (int64_t)slot * tpf) * cpw + grp;
        const int64_t row = row_ids ? row_ids[slot] : slot;
        float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
        if (c < C) {
            const char* p = reinterpret_cast<const char*>(F) + ((row * C + c) * (int64_t)HW) * sizeof(T);
            for (int base = 0; base < nv; base += UNR << g_log2) {
                V v[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int idx = base + (u << g_log2) + sub;
                    if (idx < nv)
                        v[u] = __builtin_nontemporal_load(reinterpret_cast<const V*>(p + (int64_t)idx * VB));
                    else
                        v[u] = V{};
                }
#pragma unroll
                for (int u = 0; u < UNR; u += 4) {
                    acc0 += Chunk<T, VB>::sum(v[u]);
                    if (u + 1 < UNR) acc1 += Chunk<T, VB>::sum(v[u + 1]);
                    if (u + 2 < UNR) acc2 += Chunk<T, VB>::sum(v[u + 2]);
                    if (u + 3 < UNR) acc3 += Chunk<T, VB>::sum(v[u + 3]);
                }
            }
        }
        float acc = (acc0 + acc1) + (acc2 + acc3);
        for (int off = g >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (sub == 0 && c < C) {
            const float m = acc / (float)HW;
            sv[(int64_t)frame_ids[slot] * C + c] = m;
            if (sv_out) sv_out[(int64_t)slot * C + c] = m;
        }
    }
}


// pair path: channels 2p and 2p+1 of a frame form one run of nv2 = 2*H*W*sizeof(T)/16 chunks
// (nv2 is odd); chunks below the middle one belong to channel 2p, those above to 2p+1, and the
// middle chunk holds the last 8 bytes of the first and the first 8 bytes of the second.
template <typename T, int UNR>
__global__ __launch_bounds__(256) void k_encode_pair(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    float* __restrict__ sv, float* __restrict__ sv_out, int C, int HW, int g_log2) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int n_waves = gridDim.x * (blockDim.x >> 6);
    const int g = 1 << g_log2;
    const int sub = lane & (g - 1);
    const int grp = lane >> g_log2;
    const int ppw = 64 >> g_log2;                       // channel pairs per wavefront task
    const int n_pairs = C >> 1;                         // C is even on this path
    const int tpf = (n_pairs + ppw - 1) / ppw;
    const int nv2 = (int)((int64_t)HW * sizeof(T) / 8); // 16-byte chunks per pair (odd)
    const int mid = nv2 >> 1;
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int64_t total = (int64_t)n_live * tpf;

    for (int64_t t = wave; t < total; t += n_waves) {
        const int slot = (int)(t / tpf);
        const int pr = (int)(t - (int64_t)slot * tpf) * ppw + grp;
        const int64_t row = row_ids ? row_ids[slot] : slot;
        float a0 = 0.f, a1 = 0.f, b0 = 0.f, b1 = 0.f;
        if (pr < n_pairs) {
            const char* p = reinterpret_cast<const char*>(F) + ((row * C + 2 * pr) * (int64_t)HW) * sizeof(T);
            for (int base = 0; base < nv2; base += UNR << g_log2) {
                u32x4 v[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int idx = base + (u << g_log2) + sub;
                    if (idx < nv2)
                        v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + (int64_t)idx * 16));
                    else
                        v[u] = u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int idx = base + (u << g_log2) + sub;
                    const float lo = Halves<T>::lo(v[u]), hi = Halves<T>::hi(v[u]);
                    // out-of-range chunks were loaded as zeros, so any side may take them
                    const float to_a = idx < mid ? lo + hi : (idx == mid ? lo : 0.f);
                    const float to_b = idx > mid ? lo + hi : (idx == mid ? hi : 0.f);
                    if (u & 1) { a1 += to_a; b1 += to_b; } else { a0 += to_a; b0 += to_b; }
                }
            }
        }
        float a = a0 + a1, b = b0 + b1;
        for (int off = g >> 1; off > 0; off >>= 1) {
            a += __shfl_xor(a, off, 64);
            b += __shfl_xor(b, off, 64);
        }
        if (sub == 0 && pr < n_pairs) {
            const float ma = a / (float)HW, mb = b / (float)HW;
            float* o = sv + (int64_t)frame_ids[slot] * C + 2 * pr;
            o[0] = ma; o[1] = mb;
            if (sv_out) { float* q = sv_out + (int64_t)slot * C + 2 * pr; q[0] = ma; q[1] = mb; }
        }
    }
}

// lds path.  Dynamic LDS: 4 wavefronts x (64 * HW * sizeof(T)) bytes, each a multiple of 16.
// A wavefront owns its region and its tasks (64 channels of one frame): nothing is shared between
// the wavefronts of a block, so they only order their own LDS traffic and never wait for each other.
__device__ __forceinline__ void wave_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Sum of the HW elements that start at element `first` of the wavefront's region.
template <typename T>
__device__ __forceinline__ float lds_channel_sum(const T* region, int first, int HW) {
    if constexpr (sizeof(T) == 2) {
        // two halves per 32-bit read; the first and the last word may belong to this channel only in part
        const uint32_t* wq = reinterpret_cast<const uint32_t*>(region);
        const int last = first + HW - 1;
        const int w0 = first >> 1, w1 = last >> 1;
        auto lo = [](uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u & 0xffffu)); };
        auto hi = [](uint32_t u) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(u >> 16)); };
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        uint32_t u = wq[w0];
        if (first & 1) a1 += hi(u);
        else { a0 += lo(u); if (first < last) a1 += hi(u); }
        int w = w0 + 1;
        for (; w + 2 <= w1; w += 2) {
            const uint32_t p = wq[w], q = wq[w + 1];
            a0 += lo(p); a1 += hi(p); a2 += lo(q); a3 += hi(q);
        }
        for (; w < w1; ++w) { const uint32_t p = wq[w]; a0 += lo(p); a1 += hi(p); }
        if (w1 > w0) {
            u = wq[w1];
            a0 += lo(u);
            if (last & 1) a1 += hi(u);
        }
        return (a0 + a1) + (a2 + a3);
    } else {
        const T* q = region + first;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int i = 0;
        for (; i + 4 <= HW; i += 4) {
            a0 += (float)q[i]; a1 += (float)q[i + 1]; a2 += (float)q[i + 2]; a3 += (float)q[i + 3];
        }
        for (; i < HW; ++i) a0 += (float)q[i];
        return (a0 + a1) + (a2 + a3);
    }
}

template <typename T, int UNR>
__global__ __launch_bounds__(256) void k_encode_lds(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    float* __restrict__ sv, float* __restrict__ sv_out, int C, int HW) {
    extern __shared__ u32x4 lds16[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int tile_bytes = 64 * HW * (int)sizeof(T);
    u32x4* my16 = lds16 + wave * (tile_bytes >> 4);
    T* myT = reinterpret_cast<T*>(my16);
    const int gpf = (C + 63) >> 6;                       // 64-channel groups per frame
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int64_t total = (int64_t)n_live * gpf;
    const int64_t n_waves = (int64_t)gridDim.x * 4;

    // The global loads of the next task are issued before the LDS pass over the current one, so a
    // wavefront always has loads in flight.  The launcher picks UNR so that one round of UNR loads
    // per lane covers a task: 64 * HW * sizeof(T) <= 64 * UNR * 16 bytes.
    auto fetch = [&](int64_t t, u32x4 (&v)[UNR], T& tail, int& nfull, int& nch, int& slot, int& cg) {
        slot = (int)(t / gpf);
        cg = (int)(t - (int64_t)slot * gpf);
        nch = C - cg * 64;
        if (nch > 64) nch = 64;
        const int64_t row = row_ids ? row_ids[slot] : slot;
        const T* p = F + (row * C + (int64_t)cg * 64) * HW;
        nfull = (nch * HW * (int)sizeof(T)) >> 4;
        const u32x4* p16 = reinterpret_cast<const u32x4*>(p);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int idx = u * 64 + lane;
            if (idx < nfull) v[u] = __builtin_nontemporal_load(p16 + idx);
        }
        const int done = (nfull << 4) / (int)sizeof(T);             // elements covered by whole chunks
        const int rem = nch * HW - done;                            // < 16 / sizeof(T)
        if (lane < rem) tail = p[done + lane];
    };

    u32x4 v[UNR];
    T tail = (T)0;
    int nfull = 0, nch = 0, slot = 0, cg = 0;
    int64_t t = (int64_t)blockIdx.x * 4 + wave;                     // uniform over the wavefront
    if (t < total) fetch(t, v, tail, nfull, nch, slot, cg);
    while (t < total) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int idx = u * 64 + lane;
            if (idx < nfull) my16[idx] = v[u];
        }
        {
            const int done = (nfull << 4) / (int)sizeof(T);
            if (lane < nch * HW - done) myT[done + lane] = tail;
        }
        wave_lds_order();
        const int cur_nch = nch, cur_slot = slot, cur_cg = cg;
        t += n_waves;
        if (t < total) fetch(t, v, tail, nfull, nch, slot, cg);
        if (lane < cur_nch) {
            const float m = lds_channel_sum<T>(myT, lane * HW, HW) / (float)HW;
            const int c = cur_cg * 64 + lane;
            sv[(int64_t)frame_ids[cur_slot] * C + c] = m;
            if (sv_out) sv_out[(int64_t)cur_slot * C + c] = m;
        }
        wave_lds_order();
    }
}

// Channels-last (NHWC) feature maps: a frame is H*W position rows of C channels.  A "slab" is up to 64
// consecutive 16-byte chunks of a position row (512 fp16 or 256 fp32 channels); a lane owns one
// chunk of the slab (the same channels for every position it visits) and 64 / slab-width positions
// are read per wavefront load, so loads stay contiguous.  A block handles one (frame, slab); its
// wavefronts split the positions, partial sums meet in LDS and are added in a fixed order.
template <typename T, int UNR>
__global__ __launch_bounds__(1024) void k_encode_nhwc(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    float* __restrict__ sv, float* __restrict__ sv_out, int C, int HW) {
    constexpr int E = 16 / (int)sizeof(T);               // channels per 16-byte chunk
    extern __shared__ float part[];                      // [waves][64 lanes][E]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int cpr = C / E;                               // chunks per position row (C is a multiple of E here)
    const int n_slabs = (cpr + 63) >> 6;
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int64_t total = (int64_t)n_live * n_slabs;
    for (int64_t t = blockIdx.x; t < total; t += gridDim.x) {        // uniform over the block
        const int slot = (int)(t / n_slabs);
        const int slab = (int)(t - (int64_t)slot * n_slabs);
        const int sw = cpr - slab * 64 < 64 ? cpr - slab * 64 : 64;  // chunks in this slab
        const int ppl = 64 / sw;                                     // positions per wavefront load
        const int pos_in_load = lane / sw, k = lane - pos_in_load * sw;
        const bool lane_on = pos_in_load < ppl;
        const int64_t row = row_ids ? row_ids[slot] : slot;
        const u32x4* base = reinterpret_cast<const u32x4*>(F + row * (int64_t)HW * C) + slab * 64 + k;
        // positions of this wavefront: a contiguous share of the H*W positions
        const int p_lo = (int)((int64_t)HW * wave / nw), p_hi = (int)((int64_t)HW * (wave + 1) / nw);
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;
        if (lane_on) {
            for (int p0 = p_lo + pos_in_load; p0 < p_hi; p0 += ppl * UNR) {
                u32x4 v[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int p = p0 + u * ppl;
                    if (p < p_hi) v[u] = __builtin_nontemporal_load(base + (int64_t)p * cpr);
                    else v[u] = u32x4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    if (sizeof(T) == 2) {
                        const uint32_t w4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const half2_t h = __builtin_bit_cast(half2_t, w4[q]);
                            acc[(2 * q) % E] += (float)h.x;
                            acc[(2 * q + 1) % E] += (float)h.y;
                        }
                    } else {
                        const f32x4 f = __builtin_bit_cast(f32x4, v[u]);
                        acc[0] += f.x; acc[1 % E] += f.y; acc[2 % E] += f.z; acc[3 % E] += f.w;
                    }
                }
            }
        }
#pragma unroll
        for (int e = 0; e < E; ++e) part[(wave * 64 + lane) * E + e] = lane_on ? acc[e] : 0.f;
        __syncthreads();
        // channel c of the slab = chunk k, element e: add the partial sums of every wavefront and
        // every position lane that owned chunk k, in a fixed order
        const int n_out = sw * E;
        for (int o = threadIdx.x; o < n_out; o += blockDim.x) {
            const int kk = o / E, e = o - kk * E;
            float sum = 0.f;
            for (int w = 0; w < nw; ++w)
                for (int j = 0; j < ppl; ++j) sum += part[(w * 64 + j * sw + kk) * E + e];
            const float m = sum / (float)HW;
            const int c = slab * 64 * E + o;
            sv[(int64_t)frame_ids[slot] * C + c] = m;
            if (sv_out) sv_out[(int64_t)slot * C + c] = m;
        }
        __syncthreads();
    }
}

// Fallback for channel counts that are not a multiple of a 16-byte chunk: lane = channel,
// positions walked one by one (coalesced over channels).
template <typename T>
__global__ __launch_bounds__(256) void k_encode_nhwc_scalar(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    float* __restrict__ sv, float* __restrict__ sv_out, int C, int HW) {
    int n_live = counts->n_live;
    if (n_live > max_rows) n_live = max_rows;
    const int cb = (C + 255) / 256;                      // channel blocks per frame
    const int64_t total = (int64_t)n_live * cb;
    for (int64_t t = blockIdx.x; t < total; t += gridDim.x) {
        const int slot = (int)(t / cb);
        const int c = (int)(t - (int64_t)slot * cb) * 256 + threadIdx.x;
        if (c >= C) continue;
        const int64_t row = row_ids ? row_ids[slot] : slot;
        const T* p = F + row * (int64_t)HW * C + c;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int i = 0;
        for (; i + 4 <= HW; i += 4) {
            a0 += (float)p[(int64_t)i * C]; a1 += (float)p[(int64_t)(i + 1) * C];
            a2 += (float)p[(int64_t)(i + 2) * C]; a3 += (float)p[(int64_t)(i + 3) * C];
        }
        for (; i < HW; ++i) a0 += (float)p[(int64_t)i * C];
        const float m = ((a0 + a1) + (a2 + a3)) / (float)HW;
        sv[(int64_t)frame_ids[slot] * C + c] = m;
        if (sv_out) sv_out[(int64_t)slot * C + c] = m;
    }
}

static int encode_grid(int64_t tasks_upper, int waves_per_block) {
    // enough resident wavefronts to cover HBM latency on 256 CUs, and no more blocks than tasks
    int64_t blocks = (tasks_upper + waves_per_block - 1) / waves_per_block;
    const int64_t cap = 256 * 64;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

template <typename T, int VB>
static void launch_direct(const void* fmap, int C, int HW, const int32_t* row_ids,
                          const int32_t* frame_ids, const Counts* counts, int max_rows, float* sv,
                          float* sv_out, hipStream_t st, char* name, size_t name_cap) {
    constexpr int UNR = 8;
    const int nv = (int)((int64_t)HW * sizeof(T) / VB);
    int g_log2 = 0;
    while (g_log2 < 6 && (nv + (1 << g_log2) - 1) / (1 << g_log2) > UNR) ++g_log2;
    const int cpw = 64 >> g_log2;
    const int64_t tasks = (int64_t)max_rows * ((C + cpw - 1) / cpw);
    const int grid = encode_grid(tasks, 4);
    const T* F = static_cast<const T*>(fmap);
#define SMTM_LAUNCH_DIRECT(GL)                                                                              \
    hipLaunchKernelGGL((k_encode_direct<T, VB, UNR, GL>), dim3(grid), dim3(256), 0, st, F, row_ids, frame_ids, \
                       counts, max_rows, sv, sv_out, C, HW, g_log2)
    if (VB == 16) {
        switch (g_log2) {
            case 0: SMTM_LAUNCH_DIRECT(0); break;
            case 1: SMTM_LAUNCH_DIRECT(1); break;
            case 2: SMTM_LAUNCH_DIRECT(2); break;
            case 3: SMTM_LAUNCH_DIRECT(3); break;
            case 4: SMTM_LAUNCH_DIRECT(4); break;
            case 5: SMTM_LAUNCH_DIRECT(5); break;
            default: SMTM_LAUNCH_DIRECT(6); break;
        }
    } else {
        SMTM_LAUNCH_DIRECT(-1);
    }
#undef SMTM_LAUNCH_DIRECT
    if (name) snprintf(name, name_cap, "k_encode_direct<%s,%dB,%d lanes per channel>", sizeof(T) == 2 ? "f16" : "f32", VB, 1 << g_log2);
}

template <typename T>
static void launch_pair(const void* fmap, int C, int HW, const int32_t* row_ids, const int32_t* frame_ids,
                        const Counts* counts, int max_rows, float* sv, float* sv_out, hipStream_t st, char* name,
                        size_t name_cap) {
    constexpr int UNR = 8;
    const int nv2 = (int)((int64_t)HW * sizeof(T) / 8);
    int g_log2 = 0;
    while (g_log2 < 6 && (nv2 + (1 << g_log2) - 1) / (1 << g_log2) > UNR) ++g_log2;
    const int ppw = 64 >> g_log2;
    const int64_t tasks = (int64_t)max_rows * ((C / 2 + ppw - 1) / ppw);
    const int grid = encode_grid(tasks, 4);
    hipLaunchKernelGGL((k_encode_pair<T, UNR>), dim3(grid), dim3(256), 0, st, static_cast<const T*>(fmap),
                       row_ids, frame_ids, counts, max_rows, sv, sv_out, C, HW, g_log2);
    if (name) snprintf(name, name_cap, "k_encode_pair<%s,%d lanes per pair>", sizeof(T) == 2 ? "f16" : "f32", 1 << g_log2);
}

const char* launch_encode(const void* fmap, int dtype, int C, int HW, const int32_t* row_ids,
                          const int32_t* frame_ids, const Counts* counts, int max_rows,
                          float* sv, float* sv_out, hipStream_t st, char* name, size_t name_cap) {
    const int esz = dtype == SMTM_F16 ? 2 : 4;
    const int64_t ch_bytes = (int64_t)HW * esz;
    const int64_t frame_bytes = ch_bytes * C;
    if (ch_bytes % 16 == 0) {
        if (dtype == SMTM_F16) launch_direct<_Float16, 16>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        else launch_direct<float, 16>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        return "d16";
    }
    if (ch_bytes % 8 == 0 && (C & 1) == 0) {
        if (dtype == SMTM_F16) launch_pair<_Float16>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        else launch_pair<float>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        return "pair";
    }
    if (ch_bytes % 8 == 0) {
        if (dtype == SMTM_F16) launch_direct<_Float16, 8>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        else launch_direct<float, 8>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        return "d8";
    }
    if (frame_bytes % 16 == 0 && ch_bytes <= 256) {
        const int tile_bytes = 64 * (int)ch_bytes;                 // multiple of 16 since 64*esz is
        const int gpf = (C + 63) / 64;
        int grid = encode_grid((int64_t)max_rows * gpf, 4);
        // as many blocks as stay resident at once (160 KB of LDS per CU, 8 blocks of 256 threads at most):
        // each wavefront then walks several tasks and overlaps one task's sums with the next one's loads
        int per_cu = (int)((160 * 1024) / ((size_t)tile_bytes * 4));
        if (per_cu > 8) per_cu = 8;
        if (per_cu < 1) per_cu = 1;
        if (grid > 256 * per_cu) grid = 256 * per_cu;
        const size_t lds = (size_t)tile_bytes * 4;
        // one round of UNR 16-byte loads per lane has to cover a task (64 channels): 8 up to 128-byte channels, else 16
#define SMTM_LAUNCH_LDS(T, UNR)                                                                              \
        hipLaunchKernelGGL((k_encode_lds<T, UNR>), dim3(grid), dim3(256), lds, st, static_cast<const T*>(fmap), \
                           row_ids, frame_ids, counts, max_rows, sv, sv_out, C, HW)
        if (dtype == SMTM_F16) { if (ch_bytes <= 128) SMTM_LAUNCH_LDS(_Float16, 8); else SMTM_LAUNCH_LDS(_Float16, 16); }
        else                   { if (ch_bytes <= 128) SMTM_LAUNCH_LDS(float, 8);    else SMTM_LAUNCH_LDS(float, 16); }
#undef SMTM_LAUNCH_LDS
        if (name) snprintf(name, name_cap, "k_encode_lds<%s,%d loads per lane>", dtype == SMTM_F16 ? "f16" : "f32", ch_bytes <= 128 ? 8 : 16);
        return "lds";
    }
    if (ch_bytes % 4 == 0) {
        if (dtype == SMTM_F16) launch_direct<_Float16, 4>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        else launch_direct<float, 4>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
        return "d4";
    }
    launch_direct<_Float16, 2>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, sv, sv_out, st, name, name_cap);
    return "d2";
}

const char* launch_encode_nhwc(const void* fmap, int dtype, int C, int HW, const int32_t* row_ids,
                               const int32_t* frame_ids, const Counts* counts, int max_rows,
                               float* sv, float* sv_out, hipStream_t st, char* name, size_t name_cap) {
    const int E = dtype == SMTM_F16 ? 8 : 4;
    if (C % E == 0) {
        const int cpr = C / E;
        const int n_slabs = (cpr + 63) / 64;
        const int sw = cpr < 64 ? cpr : 64, ppl = 64 / sw;
        // wavefronts per block: enough that each still issues several loads, at most 16
        int nw = HW / (ppl * 8);
        if (nw < 1) nw = 1;
        if (nw > 16) nw = 16;
        const int grid = encode_grid((int64_t)max_rows * n_slabs, 1);
        const size_t lds = (size_t)nw * 64 * E * sizeof(float);
        if (dtype == SMTM_F16)
            hipLaunchKernelGGL((k_encode_nhwc<_Float16, 8>), dim3(grid), dim3(nw * 64), lds, st,
                               static_cast<const _Float16*>(fmap), row_ids, frame_ids, counts, max_rows, sv, sv_out, C, HW);
        else
            hipLaunchKernelGGL((k_encode_nhwc<float, 8>), dim3(grid), dim3(nw * 64), lds, st,
                               static_cast<const float*>(fmap), row_ids, frame_ids, counts, max_rows, sv, sv_out, C, HW);
        if (name) snprintf(name, name_cap, "k_encode_nhwc<%s,%d wavefronts>", dtype == SMTM_F16 ? "f16" : "f32", nw);
        return "nhwc16";
    }
    const int grid = encode_grid((int64_t)max_rows * ((C + 255) / 256), 1);
    if (dtype == SMTM_F16)
        hipLaunchKernelGGL((k_encode_nhwc_scalar<_Float16>), dim3(grid), dim3(256), 0, st,
                           static_cast<const _Float16*>(fmap), row_ids, frame_ids, counts, max_rows, sv, sv_out, C, HW);
    else
        hipLaunchKernelGGL((k_encode_nhwc_scalar<float>), dim3(grid), dim3(256), 0, st,
                           static_cast<const float*>(fmap), row_ids, frame_ids, counts, max_rows, sv, sv_out, C, HW);
    if (name) snprintf(name, name_cap, "k_encode_nhwc_scalar<%s>", dtype == SMTM_F16 ? "f16" : "f32");
    return "nhwc1";
}

}  // namespace smtm
