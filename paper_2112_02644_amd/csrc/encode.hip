// Encode: semantic vector = global average pooling of each channel's H x W map
// (arXiv 2112.02644, Sec. 4.1).  The feature map is read exactly once, in place, with the
// widest loads its shape allows; sums are kept in fp32.
//
// Streaming paths for NCHW maps (a frame's C x H x W elements are contiguous):
//   flat    a wavefront takes a run of whole channels of one frame (about 6 KB, a multiple of 16 bytes) and reads
//           it as one contiguous piece, lane after lane, 16 bytes each: every load instruction covers 1 KB of
//           consecutive addresses whatever the channel length is.  Each 16-byte chunk is reduced to the sums of
//           its "units" (the largest power-of-two piece, 4..16 bytes, that never straddles two channels), the
//           unit sums go to the wavefront's own LDS region, and a group of lanes adds up each channel's units.
//   lds     channels whose length is not a multiple of 4 bytes (7x7 fp16 = 98 B): the run of 64 channels goes
//           to LDS as it is and lane c adds up channel c from LDS.
//   direct  everything else (very long channels, frames that are not a multiple of 16 bytes): a group of g lanes
//           (a power of two) owns one channel and walks it with VB-byte loads, 64/g channels per wavefront.
// In the first two the loads of a wavefront's next task are in flight while it adds up the current one.
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

// Largest |SV| of a frame (the scoring kernels scale by it).  No pass of its own and no atomics: the tasks of a
// frame (groups of channels) are split into up to kRowMaxSlots bins of consecutive tasks (with 64 bins a
// wavefront walks a few tasks, and neighbouring wavefronts read neighbouring memory at about the same time, which
// measured 6 % faster than longer walks or walks that jump through the frame), a worker (wavefront or block) takes a whole bin, keeps the largest |SV| it produced there as the bit pattern of a non-negative float
// (which orders like the value; a NaN sorts above infinity) and stores it in the frame's slot of that bin.
// Every slot of a live frame is rewritten by every encode, so nothing has to be cleared.
// Semantic vectors and these maxima are stored by live slot (dense, in the order the scoring kernel walks them);
// the worker of a frame's first bin also records the frame's slot, through which the centre update finds the
// vector of a frame later.
__device__ __forceinline__ uint32_t abs_bits(float m) { return __builtin_bit_cast(uint32_t, m) & 0x7fffffffu; }

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t bits) {
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t other = (uint32_t)__shfl_xor((int)bits, off, 64);
        bits = other > bits ? other : bits;
    }
    return bits;
}

// Live count of this launch; on the first encode of a batch also the batch's initial state (see EncodeOut).
__device__ __forceinline__ int live_count(const EncodeOut& o, const Counts* counts, int max_rows) {
    if (o.fresh) {
        const int tid = blockIdx.x * blockDim.x + threadIdx.x, stride = gridDim.x * blockDim.x;
        for (int i = tid; i < o.fresh; i += stride) {
            o.live0[i] = i;
            o.res_layer[i] = 0; o.res_label[i] = -1; o.res_tier[i] = 0;
        }
        if (tid == 0) { o.counts_w->n_live = o.fresh; o.counts_w->n_exit = 0; }
        if (tid < SMTM_MAX_EXITS * 4) o.counts_w->stats[tid >> 2][tid & 3] = 0;
        return o.fresh;
    }
    const int n = counts->n_live;
    return n > max_rows ? max_rows : n;
}

// first task of bin b when tpf tasks are split into nslots bins (nslots <= tpf, so no bin is empty)
__device__ __forceinline__ int bin_lo(int b, int tpf, int nslots) { return (int)((int64_t)b * tpf / nslots); }

static int slots_for(int tasks_per_frame) { return tasks_per_frame < kRowMaxSlots ? tasks_per_frame : kRowMaxSlots; }

template <typename T, int VB> struct Chunk;

template <> struct Chunk<_Float16, 16> {
    typedef u32x4 V;
    static __device__ __forceinline__ float sum(V v) {
        return (sum_halves(v.x) + sum_halves(v.y)) + (sum_halves(v.z) + sum_halves(v.w));
    }
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
    EncodeOut o, int C, int HW, int g_log2_arg, int nslots) {
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
    const int n_live = live_count(o, counts, max_rows);
    const int64_t total = (int64_t)n_live * nslots;     // bins

    for (int64_t bb = wave; bb < total; bb += n_waves) {
        const int slot = (int)(bb / nslots);
        const int bin = (int)(bb - (int64_t)slot * nslots);
        const int64_t row = row_ids ? row_ids[slot] : slot;
        const int frame = o.fresh ? slot : frame_ids[slot];
        uint32_t mx = 0u;
        const int t_hi = bin_lo(bin + 1, tpf, nslots);
        for (int task = bin_lo(bin, tpf, nslots); task < t_hi; ++task) {
            const int c = task * cpw + grp;
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
                o.sv[(int64_t)slot * o.ldv + c] = m;
                if (o.sv_out) o.sv_out[(int64_t)slot * C + c] = m;
                const uint32_t b = abs_bits(m);
                mx = b > mx ? b : mx;
            }
        }
        mx = wave_max_u32(mx);
        if (lane == 0) {
            o.rowmax[(int64_t)slot * kRowMaxSlots + bin] = mx;
            if (bin == 0) o.slot_of[frame] = slot;
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
    EncodeOut o, int C, int HW, int nslots) {
    extern __shared__ u32x4 lds16[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int tile_bytes = 64 * HW * (int)sizeof(T);
    u32x4* my16 = lds16 + wave * (tile_bytes >> 4);
    T* myT = reinterpret_cast<T*>(my16);
    const int gpf = (C + 63) >> 6;                       // tasks (64-channel groups) per frame
    const int n_live = live_count(o, counts, max_rows);
    const int64_t total = (int64_t)n_live * nslots;      // bins
    const int64_t n_waves = (int64_t)gridDim.x * 4;

    // A wavefront walks its bins (bb, bb + n_waves, ...) and inside a bin the bin's tasks.  The global loads of
    // the next task are issued before the LDS pass over the current one, so a wavefront always has loads in
    // flight.  The launcher picks UNR so that one round of UNR loads per lane covers a task:
    // 64 * HW * sizeof(T) <= 64 * UNR * 16 bytes.
    struct Task { int slot, bin, cg, hi, frame, nch, nfull; };
    auto open_bin = [&](int64_t bb, Task& k) {           // first task of bin bb
        k.slot = (int)(bb / nslots);
        k.bin = (int)(bb - (int64_t)k.slot * nslots);
        k.cg = bin_lo(k.bin, gpf, nslots);
        k.hi = bin_lo(k.bin + 1, gpf, nslots);
        k.frame = o.fresh ? k.slot : frame_ids[k.slot];
    };
    auto fetch = [&](Task& k, u32x4 (&v)[UNR], T& tail) {
        k.nch = C - k.cg * 64;
        if (k.nch > 64) k.nch = 64;
        const int64_t row = row_ids ? row_ids[k.slot] : k.slot;
        const T* p = F + (row * C + (int64_t)k.cg * 64) * HW;
        k.nfull = (k.nch * HW * (int)sizeof(T)) >> 4;
        const u32x4* p16 = reinterpret_cast<const u32x4*>(p);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int idx = u * 64 + lane;
            if (idx < k.nfull) v[u] = __builtin_nontemporal_load(p16 + idx);
        }
        const int done = (k.nfull << 4) / (int)sizeof(T);           // elements covered by whole chunks
        const int rem = k.nch * HW - done;                          // < 16 / sizeof(T)
        if (lane < rem) tail = p[done + lane];
    };

    u32x4 v[UNR];
    T tail = (T)0;
    Task nxt = {};
    int64_t bb = (int64_t)blockIdx.x * 4 + wave;                    // uniform over the wavefront
    bool more = bb < total;
    if (more) { open_bin(bb, nxt); fetch(nxt, v, tail); }
    uint32_t mx = 0u;
    while (more) {
        const Task cur = nxt;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int idx = u * 64 + lane;
            if (idx < cur.nfull) my16[idx] = v[u];
        }
        {
            const int done = (cur.nfull << 4) / (int)sizeof(T);
            if (lane < cur.nch * HW - done) myT[done + lane] = tail;
        }
        wave_lds_order();
        // next task: the next one of this bin, else the first one of the wavefront's next bin
        const bool last_of_bin = cur.cg + 1 >= cur.hi;
        if (!last_of_bin) { nxt.cg = cur.cg + 1; }
        else { bb += n_waves; more = bb < total; if (more) open_bin(bb, nxt); }
        if (more) fetch(nxt, v, tail);
        if (lane < cur.nch) {
            const float m = lds_channel_sum<T>(myT, lane * HW, HW) / (float)HW;
            const int c = cur.cg * 64 + lane;
            o.sv[(int64_t)cur.slot * o.ldv + c] = m;
            if (o.sv_out) o.sv_out[(int64_t)cur.slot * C + c] = m;
            const uint32_t b = abs_bits(m);
            mx = b > mx ? b : mx;
        }
        if (last_of_bin) {
            mx = wave_max_u32(mx);
            if (lane == 0) {
                o.rowmax[(int64_t)cur.slot * kRowMaxSlots + cur.bin] = mx;
                if (cur.bin == 0) o.slot_of[cur.frame] = cur.slot;
            }
            mx = 0u;
        }
        wave_lds_order();
    }
}

// flat path.  UB = unit bytes (4, 8 or 16), UNR = 16-byte loads per lane that cover a task.
// Dynamic LDS: 4 wavefronts x (chunks per task) x (16 / UB) floats.
template <typename T, int UB> struct Units;               // sums of the 16 / UB units of a 16-byte chunk
template <> struct Units<_Float16, 16> {
    static __device__ __forceinline__ void put(float* dst, u32x4 v) {
        *dst = (sum_halves(v.x) + sum_halves(v.y)) + (sum_halves(v.z) + sum_halves(v.w));
    }
};
template <> struct Units<_Float16, 8> {
    static __device__ __forceinline__ void put(float* dst, u32x4 v) {
        *reinterpret_cast<f32x2*>(dst) = f32x2{sum_halves(v.x) + sum_halves(v.y), sum_halves(v.z) + sum_halves(v.w)};
    }
};
template <> struct Units<_Float16, 4> {
    static __device__ __forceinline__ void put(float* dst, u32x4 v) {
        *reinterpret_cast<f32x4*>(dst) = f32x4{sum_halves(v.x), sum_halves(v.y), sum_halves(v.z), sum_halves(v.w)};
    }
};
template <> struct Units<float, 16> {
    static __device__ __forceinline__ void put(float* dst, u32x4 v) {
        const f32x4 f = __builtin_bit_cast(f32x4, v);
        *dst = (f.x + f.y) + (f.z + f.w);
    }
};
template <> struct Units<float, 8> {
    static __device__ __forceinline__ void put(float* dst, u32x4 v) {
        const f32x4 f = __builtin_bit_cast(f32x4, v);
        *reinterpret_cast<f32x2*>(dst) = f32x2{f.x + f.y, f.z + f.w};
    }
};
template <> struct Units<float, 4> {
    static __device__ __forceinline__ void put(float* dst, u32x4 v) { *reinterpret_cast<f32x4*>(dst) = __builtin_bit_cast(f32x4, v); }
};

template <typename T, int UB, int UNR>
__global__ __launch_bounds__(256) void k_encode_flat(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    EncodeOut o, int C, int HW, int cps, int lpc_log2, int region_floats, int nslots) {
    constexpr int UPC16 = 16 / UB;                       // units per 16-byte chunk
    extern __shared__ __attribute__((aligned(16))) float lds_units[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float* my = lds_units + wave * region_floats;
    const int upc = HW * (int)sizeof(T) / UB;            // units per channel
    const int tpf = (C + cps - 1) / cps;                 // tasks (runs of cps channels) per frame
    const int lpc = 1 << lpc_log2;                       // lanes that share a channel's units (cps * lpc <= 64)
    const int ch = lane >> lpc_log2, part = lane & (lpc - 1);
    const int n_live = live_count(o, counts, max_rows);
    const int64_t total = (int64_t)n_live * nslots;      // bins
    const int64_t n_waves = (int64_t)gridDim.x * 4;

    struct Task { int slot, bin, task, hi, frame, nch, nchunks; };
    auto open_bin = [&](int64_t bb, Task& k) {           // first task of bin bb
        k.slot = (int)(bb / nslots);
        k.bin = (int)(bb - (int64_t)k.slot * nslots);
        k.task = bin_lo(k.bin, tpf, nslots);
        k.hi = bin_lo(k.bin + 1, tpf, nslots);
        k.frame = o.fresh ? k.slot : frame_ids[k.slot];
    };
    auto fetch = [&](Task& k, u32x4 (&v)[UNR]) {
        k.nch = C - k.task * cps;
        if (k.nch > cps) k.nch = cps;
        const int64_t row = row_ids ? row_ids[k.slot] : k.slot;
        const u32x4* p16 = reinterpret_cast<const u32x4*>(F + (row * C + (int64_t)k.task * cps) * HW);
        k.nchunks = (k.nch * HW * (int)sizeof(T)) >> 4;  // exact: the run is a multiple of 16 bytes
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int idx = u * 64 + lane;
            if (idx < k.nchunks) v[u] = __builtin_nontemporal_load(p16 + idx);
        }
    };

    u32x4 v[UNR];
    Task nxt = {};
    int64_t bb = (int64_t)blockIdx.x * 4 + wave;         // uniform over the wavefront
    bool more = bb < total;
    if (more) { open_bin(bb, nxt); fetch(nxt, v); }
    uint32_t mx = 0u;
    while (more) {
        const Task cur = nxt;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int idx = u * 64 + lane;
            if (idx < cur.nchunks) Units<T, UB>::put(my + idx * UPC16, v[u]);
        }
        wave_lds_order();
        // next task: the next one of this bin, else the first one of the wavefront's next bin
        const bool last_of_bin = cur.task + 1 >= cur.hi;
        if (!last_of_bin) { nxt.task = cur.task + 1; }
        else { bb += n_waves; more = bb < total; if (more) open_bin(bb, nxt); }
        if (more) fetch(nxt, v);
        // channel ch of the run: its units, every lpc-th one starting at `part`, then the lpc lanes combine
        float a0 = 0.f, a1 = 0.f;
        if (ch < cur.nch) {
            const float* q = my + ch * upc;
            int i = part;
            for (; i + lpc < upc; i += 2 * lpc) { a0 += q[i]; a1 += q[i + lpc]; }
            if (i < upc) a0 += q[i];
        }
        float acc = a0 + a1;
        for (int off = lpc >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (part == 0 && ch < cur.nch) {
            const float m = acc / (float)HW;
            const int c = cur.task * cps + ch;
            o.sv[(int64_t)cur.slot * o.ldv + c] = m;
            if (o.sv_out) o.sv_out[(int64_t)cur.slot * C + c] = m;
            const uint32_t b = abs_bits(m);
            mx = b > mx ? b : mx;
        }
        if (last_of_bin) {
            mx = wave_max_u32(mx);
            if (lane == 0) {
                o.rowmax[(int64_t)cur.slot * kRowMaxSlots + cur.bin] = mx;
                if (cur.bin == 0) o.slot_of[cur.frame] = cur.slot;
            }
            mx = 0u;
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
    EncodeOut o, int C, int HW, int nslots) {
    constexpr int E = 16 / (int)sizeof(T);               // channels per 16-byte chunk
    extern __shared__ float part[];                      // [waves][64 lanes][E]
    __shared__ uint32_t wmax[16];                        // largest |SV| bits per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int cpr = C / E;                               // chunks per position row (C is a multiple of E here)
    const int n_slabs = (cpr + 63) >> 6;                 // tasks per frame
    const int n_live = live_count(o, counts, max_rows);
    const int64_t total = (int64_t)n_live * nslots;      // bins
    for (int64_t bb = blockIdx.x; bb < total; bb += gridDim.x) {     // uniform over the block
      const int slot = (int)(bb / nslots);
      const int bin = (int)(bb - (int64_t)slot * nslots);
      const int frame = o.fresh ? slot : frame_ids[slot];
      uint32_t mx = 0u;
      const int s_hi = bin_lo(bin + 1, n_slabs, nslots);
      for (int slab = bin_lo(bin, n_slabs, nslots); slab < s_hi; ++slab) {
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
        for (int q = threadIdx.x; q < n_out; q += blockDim.x) {
            const int kk = q / E, e = q - kk * E;
            float sum = 0.f;
            for (int w = 0; w < nw; ++w)
                for (int j = 0; j < ppl; ++j) sum += part[(w * 64 + j * sw + kk) * E + e];
            const float m = sum / (float)HW;
            const int c = slab * 64 * E + q;
            o.sv[(int64_t)slot * o.ldv + c] = m;
            if (o.sv_out) o.sv_out[(int64_t)slot * C + c] = m;
            const uint32_t b = abs_bits(m);
            mx = b > mx ? b : mx;
        }
        __syncthreads();
      }
      // the block's largest |SV| of the bin: per wavefront, then over the wavefronts
      mx = wave_max_u32(mx);
      if (lane == 0) wmax[wave] = mx;
      __syncthreads();
      if (threadIdx.x == 0) {
          uint32_t m = 0u;
          for (int w = 0; w < nw; ++w) m = wmax[w] > m ? wmax[w] : m;
          o.rowmax[(int64_t)slot * kRowMaxSlots + bin] = m;
          if (bin == 0) o.slot_of[frame] = slot;
      }
      __syncthreads();
    }
}

// Channels-last maps with few positions (7x7, 14x14) and wide rows: a wavefront takes a (frame, slab of 64
// chunks) alone and walks the positions, 1 KB per load, UNR loads in flight, a lane adding up its own 16-byte chunk
// of channels in registers.  No LDS and no barrier; the slab is one bin of the frame's partial maxima.
template <typename T, int UNR>
__global__ __launch_bounds__(256) void k_encode_nhwc_wave(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    EncodeOut o, int C, int HW) {
    constexpr int E = 16 / (int)sizeof(T);               // channels per 16-byte chunk
    const int lane = threadIdx.x & 63;
    const int cpr = C / E;                               // chunks per position row, a multiple of 64 here
    const int n_slabs = cpr >> 6;                        // tasks per frame = bins per frame
    const int n_live = live_count(o, counts, max_rows);
    const int64_t total = (int64_t)n_live * n_slabs;
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    for (int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); t < total; t += n_waves) {
        const int slot = (int)(t / n_slabs);
        const int slab = (int)(t - (int64_t)slot * n_slabs);
        const int frame = o.fresh ? slot : frame_ids[slot];
        const int64_t row = row_ids ? row_ids[slot] : slot;
        const u32x4* base = reinterpret_cast<const u32x4*>(F + row * (int64_t)HW * C) + slab * 64 + lane;
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;
        for (int p0 = 0; p0 < HW; p0 += UNR) {
            u32x4 v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                v[u] = p0 + u < HW ? __builtin_nontemporal_load(base + (int64_t)(p0 + u) * cpr) : u32x4{0u, 0u, 0u, 0u};
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
        uint32_t mx = 0u;
        const int c0 = (slab * 64 + lane) * E;
        float m[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            m[e] = acc[e] / (float)HW;
            const uint32_t b = abs_bits(m[e]);
            mx = b > mx ? b : mx;
        }
        float* dst = o.sv + (int64_t)slot * o.ldv + c0;               // 16-byte aligned: ldv and c0 are multiples of 4
#pragma unroll
        for (int e = 0; e < E; e += 4) *reinterpret_cast<f32x4*>(dst + e) = f32x4{m[e], m[e + 1], m[e + 2], m[e + 3]};
        if (o.sv_out) {
            float* q = o.sv_out + (int64_t)slot * C + c0;
#pragma unroll
            for (int e = 0; e < E; ++e) q[e] = m[e];
        }
        mx = wave_max_u32(mx);
        if (lane == 0) {
            o.rowmax[(int64_t)slot * kRowMaxSlots + slab] = mx;
            if (slab == 0) o.slot_of[frame] = slot;
        }
    }
}

// Fallback for channel counts that are not a multiple of a 16-byte chunk: lane = channel,
// positions walked one by one (coalesced over channels).
template <typename T>
__global__ __launch_bounds__(256) void k_encode_nhwc_scalar(
    const T* __restrict__ F, const int32_t* __restrict__ row_ids,
    const int32_t* __restrict__ frame_ids, const Counts* __restrict__ counts, int max_rows,
    EncodeOut o, int C, int HW, int nslots) {
    __shared__ uint32_t wmax[4];
    const int n_live = live_count(o, counts, max_rows);
    const int cb = (C + 255) / 256;                      // tasks (256-channel blocks) per frame
    const int64_t total = (int64_t)n_live * nslots;      // bins
    for (int64_t bb = blockIdx.x; bb < total; bb += gridDim.x) {     // uniform over the block
        const int slot = (int)(bb / nslots);
        const int bin = (int)(bb - (int64_t)slot * nslots);
        const int frame = o.fresh ? slot : frame_ids[slot];
        const int64_t row = row_ids ? row_ids[slot] : slot;
        uint32_t mx = 0u;
        const int t_hi = bin_lo(bin + 1, cb, nslots);
        for (int task = bin_lo(bin, cb, nslots); task < t_hi; ++task) {
            const int c = task * 256 + threadIdx.x;
            if (c < C) {
                const T* p = F + row * (int64_t)HW * C + c;
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
                int i = 0;
                for (; i + 4 <= HW; i += 4) {
                    a0 += (float)p[(int64_t)i * C]; a1 += (float)p[(int64_t)(i + 1) * C];
                    a2 += (float)p[(int64_t)(i + 2) * C]; a3 += (float)p[(int64_t)(i + 3) * C];
                }
                for (; i < HW; ++i) a0 += (float)p[(int64_t)i * C];
                const float m = ((a0 + a1) + (a2 + a3)) / (float)HW;
                o.sv[(int64_t)slot * o.ldv + c] = m;
                if (o.sv_out) o.sv_out[(int64_t)slot * C + c] = m;
                const uint32_t b = abs_bits(m);
                mx = b > mx ? b : mx;
            }
        }
        mx = wave_max_u32(mx);
        if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = mx;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t m = wmax[0];
            for (int w = 1; w < 4; ++w) m = wmax[w] > m ? wmax[w] : m;
            o.rowmax[(int64_t)slot * kRowMaxSlots + bin] = m;
            if (bin == 0) o.slot_of[frame] = slot;
        }
        __syncthreads();
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
                          const int32_t* frame_ids, const Counts* counts, int max_rows, const EncodeOut& out,
                          hipStream_t st, char* name, size_t name_cap, int* slots) {
    constexpr int UNR = 8;
    const int nv = (int)((int64_t)HW * sizeof(T) / VB);
    int g_log2 = 0;
    while (g_log2 < 6 && (nv + (1 << g_log2) - 1) / (1 << g_log2) > UNR) ++g_log2;
    const int cpw = 64 >> g_log2;
    const int nslots = slots_for((C + cpw - 1) / cpw);
    *slots = nslots;
    const int grid = encode_grid((int64_t)max_rows * nslots, 4);
    const T* F = static_cast<const T*>(fmap);
#define SMTM_LAUNCH_DIRECT(GL)                                                                              \
    hipLaunchKernelGGL((k_encode_direct<T, VB, UNR, GL>), dim3(grid), dim3(256), 0, st, F, row_ids, frame_ids, \
                       counts, max_rows, out, C, HW, g_log2, nslots)
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

// flat path: cps channels per task, a power of two times the fewest channels whose bytes are a multiple of 16,
// as many as keep a task within 8 loads per lane (8 KB).  Returns false when the shape does not fit this path.
template <typename T>
static bool launch_flat(const void* fmap, int C, int HW, const int32_t* row_ids, const int32_t* frame_ids,
                        const Counts* counts, int max_rows, const EncodeOut& out, hipStream_t st, char* name,
                        size_t name_cap, int* slots) {
    constexpr int UNR = 8;
    const int64_t ch_bytes = (int64_t)HW * sizeof(T);
    int ub = 16;
    while (ub > 4 && ch_bytes % ub != 0) ub >>= 1;
    if (ch_bytes % ub != 0) return false;                // channels that are not a multiple of 4 bytes
    int cps = 16 / ub;                                   // fewest channels that make a multiple of 16 bytes
    if (C % cps != 0 || cps * ch_bytes > 64 * UNR * 16) return false;
    while (cps * 2 <= 64 && cps * 2 * ch_bytes <= 6272 && cps * 2 <= C) cps *= 2;   // 6272 B = 49 cache lines of 128 B
    // a task of one long channel gains nothing from the LDS pass: the direct path adds it up in registers
    if (cps == 1 && ch_bytes % 16 == 0 && ch_bytes >= 4096) return false;
    int lpc_log2 = 0;
    while ((cps << (lpc_log2 + 1)) <= 64) ++lpc_log2;
    const int task_chunks = (int)(cps * ch_bytes / 16);
    const int region_floats = task_chunks * (16 / ub);
    const int nslots = slots_for((C + cps - 1) / cps);
    *slots = nslots;
    const size_t lds = (size_t)region_floats * sizeof(float) * 4;
    int grid = encode_grid((int64_t)max_rows * nslots, 4);
    const T* F = static_cast<const T*>(fmap);
#define SMTM_LAUNCH_FLAT(UB)                                                                                        \
    hipLaunchKernelGGL((k_encode_flat<T, UB, UNR>), dim3(grid), dim3(256), lds, st, F, row_ids, frame_ids, counts,  \
                       max_rows, out, C, HW, cps, lpc_log2, region_floats, nslots)
    if (ub == 16) SMTM_LAUNCH_FLAT(16);
    else if (ub == 8) SMTM_LAUNCH_FLAT(8);
    else SMTM_LAUNCH_FLAT(4);
#undef SMTM_LAUNCH_FLAT
    if (name) snprintf(name, name_cap, "k_encode_flat<%s,%dB units,%d channels per task>", sizeof(T) == 2 ? "f16" : "f32", ub, cps);
    return true;
}

const char* launch_encode(const void* fmap, int dtype, int C, int HW, const int32_t* row_ids,
                          const int32_t* frame_ids, const Counts* counts, int max_rows,
                          const EncodeOut& out, hipStream_t st, char* name, size_t name_cap, int* slots) {
    const int esz = dtype == SMTM_F16 ? 2 : 4;
    const int64_t ch_bytes = (int64_t)HW * esz;
    const int64_t frame_bytes = ch_bytes * C;
    if (dtype == SMTM_F16 ? launch_flat<_Float16>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots)
                          : launch_flat<float>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots))
        return "flat";
    if (ch_bytes % 16 == 0) {
        if (dtype == SMTM_F16) launch_direct<_Float16, 16>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
        else launch_direct<float, 16>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
        return "d16";
    }
    if (ch_bytes % 8 == 0) {
        if (dtype == SMTM_F16) launch_direct<_Float16, 8>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
        else launch_direct<float, 8>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
        return "d8";
    }
    if (frame_bytes % 16 == 0 && ch_bytes <= 256) {
        const int tile_bytes = 64 * (int)ch_bytes;                 // multiple of 16 since 64*esz is
        const int gpf = (C + 63) / 64;
        const int nslots = slots_for(gpf);
        *slots = nslots;
        // one block per four bins (measured against a grid cut down to what stays resident: 38 against 41 us for
        // 1024 frames of 2048 x 7 x 7; the dispatcher evens out the tail better than long walks per wavefront)
        const int grid = encode_grid((int64_t)max_rows * nslots, 4);
        const size_t lds = (size_t)tile_bytes * 4;
        // one round of UNR 16-byte loads per lane has to cover a task (64 channels): 8 up to 128-byte channels, else 16
#define SMTM_LAUNCH_LDS(T, UNR)                                                                              \
        hipLaunchKernelGGL((k_encode_lds<T, UNR>), dim3(grid), dim3(256), lds, st, static_cast<const T*>(fmap), \
                           row_ids, frame_ids, counts, max_rows, out, C, HW, nslots)
        if (dtype == SMTM_F16) { if (ch_bytes <= 128) SMTM_LAUNCH_LDS(_Float16, 8); else SMTM_LAUNCH_LDS(_Float16, 16); }
        else                   { if (ch_bytes <= 128) SMTM_LAUNCH_LDS(float, 8);    else SMTM_LAUNCH_LDS(float, 16); }
#undef SMTM_LAUNCH_LDS
        if (name) snprintf(name, name_cap, "k_encode_lds<%s,%d loads per lane>", dtype == SMTM_F16 ? "f16" : "f32", ch_bytes <= 128 ? 8 : 16);
        return "lds";
    }
    if (ch_bytes % 4 == 0) {
        if (dtype == SMTM_F16) launch_direct<_Float16, 4>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
        else launch_direct<float, 4>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
        return "d4";
    }
    launch_direct<_Float16, 2>(fmap, C, HW, row_ids, frame_ids, counts, max_rows, out, st, name, name_cap, slots);
    return "d2";
}

const char* launch_encode_nhwc(const void* fmap, int dtype, int C, int HW, const int32_t* row_ids,
                               const int32_t* frame_ids, const Counts* counts, int max_rows,
                               const EncodeOut& out, hipStream_t st, char* name, size_t name_cap, int* slots) {
    const int E = dtype == SMTM_F16 ? 8 : 4;
    if (C % E == 0) {
        const int cpr = C / E;
        const int n_slabs = (cpr + 63) / 64;
        if (cpr % 64 == 0 && n_slabs <= kRowMaxSlots && HW <= 256 && (int64_t)max_rows * n_slabs >= 2048) {
            // few positions, full slabs, enough (frame, slab) pairs to give every SIMD several wavefronts
            *slots = n_slabs;
            const int grid = encode_grid((int64_t)max_rows * n_slabs, 4);
            // loads in flight per lane: 49 positions in two rounds of 25, more positions in rounds of 16
#define SMTM_LAUNCH_NHWC_WAVE(T, UNR)                                                                       \
            hipLaunchKernelGGL((k_encode_nhwc_wave<T, UNR>), dim3(grid), dim3(256), 0, st,                  \
                               static_cast<const T*>(fmap), row_ids, frame_ids, counts, max_rows, out, C, HW)
            if (dtype == SMTM_F16) { if (HW <= 50) SMTM_LAUNCH_NHWC_WAVE(_Float16, 25); else SMTM_LAUNCH_NHWC_WAVE(_Float16, 16); }
            else                   { if (HW <= 50) SMTM_LAUNCH_NHWC_WAVE(float, 25);    else SMTM_LAUNCH_NHWC_WAVE(float, 16); }
#undef SMTM_LAUNCH_NHWC_WAVE
            if (name) snprintf(name, name_cap, "k_encode_nhwc_wave<%s>", dtype == SMTM_F16 ? "f16" : "f32");
            return "nhwcw";
        }
        const int sw = cpr < 64 ? cpr : 64, ppl = 64 / sw;
        // wavefronts per block: enough that each still issues several loads, at most 16
        int nw = HW / (ppl * 8);
        if (nw < 1) nw = 1;
        if (nw > 16) nw = 16;
        const int nslots = slots_for(n_slabs);
        *slots = nslots;
        const int grid = encode_grid((int64_t)max_rows * nslots, 1);
        const size_t lds = (size_t)nw * 64 * E * sizeof(float);
        if (dtype == SMTM_F16)
            hipLaunchKernelGGL((k_encode_nhwc<_Float16, 8>), dim3(grid), dim3(nw * 64), lds, st,
                               static_cast<const _Float16*>(fmap), row_ids, frame_ids, counts, max_rows, out, C, HW, nslots);
        else
            hipLaunchKernelGGL((k_encode_nhwc<float, 8>), dim3(grid), dim3(nw * 64), lds, st,
                               static_cast<const float*>(fmap), row_ids, frame_ids, counts, max_rows, out, C, HW, nslots);
        if (name) snprintf(name, name_cap, "k_encode_nhwc<%s,%d wavefronts>", dtype == SMTM_F16 ? "f16" : "f32", nw);
        return "nhwc16";
    }
    const int nslots = slots_for((C + 255) / 256);
    *slots = nslots;
    const int grid = encode_grid((int64_t)max_rows * nslots, 1);
    if (dtype == SMTM_F16)
        hipLaunchKernelGGL((k_encode_nhwc_scalar<_Float16>), dim3(grid), dim3(256), 0, st,
                           static_cast<const _Float16*>(fmap), row_ids, frame_ids, counts, max_rows, out, C, HW, nslots);
    else
        hipLaunchKernelGGL((k_encode_nhwc_scalar<float>), dim3(grid), dim3(256), 0, st,
                           static_cast<const float*>(fmap), row_ids, frame_ids, counts, max_rows, out, C, HW, nslots);
    if (name) snprintf(name, name_cap, "k_encode_nhwc_scalar<%s>", dtype == SMTM_F16 ? "f16" : "f32");
    return "nhwc1";
}

}  // namespace smtm

