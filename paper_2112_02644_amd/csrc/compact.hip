// Exit and compact: frames released at an exit point leave the batch, the others continue
// (arXiv 2112.02644, Sec. 1 "skips the rest layers", Sec. 5 last paragraph).  For a batch this
// is a stable partition of the live list: wavefront ballot + popcount prefix inside a
// wavefront, an LDS scan across the wavefronts of one block, running bases across chunks.
// No atomics decide positions, so the lists come out in ascending frame id on every run.
#include "internal.h"
#include "decide.h"

namespace smtm {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Start of a batch: identity live list, per-frame results and counters cleared.  The accumulated similarities
// are not touched: the first lookup of the batch overwrites them.
__global__ __launch_bounds__(256) void k_begin_batch(int batch, int32_t* __restrict__ live,
                                                     int32_t* __restrict__ res_layer,
                                                     int32_t* __restrict__ res_label,
                                                     int32_t* __restrict__ res_tier,
                                                     Counts* __restrict__ counts) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    const int stride = gridDim.x * blockDim.x;
    for (int i = tid; i < batch; i += stride) {
        live[i] = i;
        res_layer[i] = 0; res_label[i] = -1; res_tier[i] = 0;
    }
    if (tid == 0) { counts->n_live = batch; counts->n_exit = 0; }
    if (tid < SMTM_MAX_EXITS * 4) counts->stats[tid >> 2][tid & 3] = 0;
}

void launch_begin_batch(int batch, int32_t* live, int32_t* res_layer, int32_t* res_label, int32_t* res_tier,
                        Counts* counts, hipStream_t st) {
    int grid = (batch + 255) / 256;
    if (grid > 256) grid = 256;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(k_begin_batch, dim3(grid), dim3(256), 0, st, batch, live, res_layer, res_label, res_tier,
                       counts);
}

// Stable partition of the live list by one block: wavefront ballot + popcount prefix, an LDS scan
// over the block's wavefronts, running bases across chunks of the list.
// With `g` the decisions are not read from memory but made here, from the per-tile results of the scoring
// kernel (and written out, with the top-2 values, as the stand-alone decision kernel would).
template <int NW>                                        // wavefronts in the block
__device__ __forceinline__ void compact_block(const CompactArgs& a, const DecideArgs* g) {
    __shared__ int w_exit[NW], w_t1[NW];
    __shared__ int base_exit, base_t1;
    constexpr int BS = NW * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The first chunk's entries are fetched together with the live count (all of it was written by the
    // kernel before; fetched one after the other it would cost three round trips).  The lists have
    // max_rows entries.
    int n_live = a.counts->n_live;
    int d_nx = 0, frame_nx = 0, lab_nx = -1;             // what the next chunk's slot of this thread will need
    SlotTop2 m_nx = {};
    auto prefetch = [&](int slot) {                      // loads only; any slot of the batch is readable
        if (slot < a.max_rows) {
            frame_nx = a.frame_ids[slot];
            if (!g) { d_nx = a.decision[slot]; lab_nx = a.label[slot]; }
            else m_nx = merge_slot(*g, slot);
        }
    };
    prefetch(tid);
    asm volatile("" : "+v"(d_nx), "+v"(frame_nx), "+v"(lab_nx), "+s"(n_live));   // issued before any is waited for
    if (tid == 0) { base_exit = 0; base_t1 = 0; }
    __syncthreads();
    for (int c0 = 0; c0 < n_live; c0 += BS) {            // uniform over the block
        const int slot = c0 + tid;
        const bool valid = slot < n_live;
        int d = d_nx, lab = lab_nx;
        const int frame = frame_nx;
        const SlotTop2 m = m_nx;
        if (c0 + BS < n_live) prefetch(slot + BS);       // the next chunk's loads fly during this chunk's scan
        if (valid) {
            if (g) { const SlotDecision sd = finish_slot(*g, slot, m); d = sd.d; lab = sd.label; }
        } else { d = 0; lab = -1; }
        const bool ex = valid && d != 0;
        const unsigned long long m_ex = __ballot(ex);
        const unsigned long long m_t1 = __ballot(valid && d == 1);
        const unsigned long long below = (1ull << lane) - 1ull;
        const int pre_ex = __popcll(m_ex & below);
        if (lane == 0) { w_exit[wave] = __popcll(m_ex); w_t1[wave] = __popcll(m_t1); }
        __syncthreads();
        int off_ex = 0, tot_ex = 0, tot_t1 = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            if (w < wave) off_ex += w_exit[w];
            tot_ex += w_exit[w]; tot_t1 += w_t1[w];
        }
        const int be = base_exit;
        if (valid) {
            if (ex) {
                const int pos = be + off_ex + pre_ex;
                if (a.exit_ids) a.exit_ids[pos] = frame;
                if (a.exit_labels) a.exit_labels[pos] = lab;
                if (a.exit_tier) a.exit_tier[pos] = d;
                a.res_layer[frame] = a.exit_index; a.res_label[frame] = lab; a.res_tier[frame] = d;
            } else {
                // survivors before this slot = slots before it minus exits before it
                const int pos = slot - (be + off_ex + pre_ex);
                a.next_ids[pos] = frame;
                a.next_slots[pos] = slot;
                if (a.live_ids_user) a.live_ids_user[pos] = frame;
            }
        }
        __syncthreads();
        if (tid == 0) { base_exit = be + tot_ex; base_t1 += tot_t1; }
        __syncthreads();
    }
    if (tid == 0) {
        const int ne = base_exit, nl = n_live - base_exit;
        a.counts->stats[a.exit_index - 1][0] = n_live;
        a.counts->stats[a.exit_index - 1][1] = base_t1;
        a.counts->stats[a.exit_index - 1][2] = ne - base_t1;
        a.counts->n_exit = ne;
        a.counts->n_live = nl;
        if (a.n_exit_dev) *a.n_exit_dev = ne;
        if (a.n_live_dev) *a.n_live_dev = nl;
    }
}

// One block of 1024 threads (16 wavefronts) walks the live list in chunks of 1024 slots.
__global__ __launch_bounds__(1024) void k_compact(CompactArgs a) {
    compact_block<16>(a, nullptr);
}

void launch_compact(const CompactArgs& args, hipStream_t st) {
    hipLaunchKernelGGL(k_compact, dim3(1), dim3(1024), 0, st, args);
}

// Decision and compaction in one launch: each thread first merges its slot's per-tile results and applies
// the exit rule, then the block partitions the live list.
__global__ __launch_bounds__(1024) void k_decide_compact(DecideArgs g, CompactArgs a) {
    compact_block<16>(a, &g);
}

void launch_decide_compact(const DecideArgs& g, const CompactArgs& args, hipStream_t st) {
    hipLaunchKernelGGL(k_decide_compact, dim3(1), dim3(1024), 0, st, g, args);
}

// Gather of the survivors' feature-map rows: new slot s copies the row that old slot
// next_slots[s] read.  VB bytes per lane per access.
template <typename V>
__global__ __launch_bounds__(256) void k_gather_rows(const char* __restrict__ src,
                                                     const int32_t* __restrict__ row_ids,
                                                     const int32_t* __restrict__ next_slots,
                                                     const Counts* __restrict__ counts, int max_rows,
                                                     char* __restrict__ dst, int64_t row_bytes) {
    int n_live = counts->n_live;                          // survivors (k_compact has run)
    if (n_live > max_rows) n_live = max_rows;
    const int64_t per_row = row_bytes / (int64_t)sizeof(V);
    for (int s = blockIdx.y; s < n_live; s += gridDim.y) {
        const int old_slot = next_slots[s];
        const int64_t row = row_ids ? row_ids[old_slot] : old_slot;
        const V* from = reinterpret_cast<const V*>(src + row * row_bytes);
        V* to = reinterpret_cast<V*>(dst + (int64_t)s * row_bytes);
        const int64_t step = (int64_t)gridDim.x * blockDim.x;
        int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
        for (; q < per_row; q += step) __builtin_nontemporal_store(__builtin_nontemporal_load(from + q), to + q);
    }
}

void launch_gather_rows(const void* src, const int32_t* row_ids, const int32_t* next_slots,
                        const Counts* counts, int max_rows, void* dst, int64_t row_bytes,
                        hipStream_t st) {
    // Many small blocks copy faster than few large ones: a thread moves one piece of a row at a time and a column
    // of blocks walks the rows, a quarter of the possible survivors per grid row (blocks that find no row left
    // still wait for the live count, so a grid row per possible survivor costs more than it gains when few
    // frames survive).  708 rows of 1.6 MB: 6.4 TB/s read + write against 5.8 TB/s for 4096 blocks with four
    // loads in flight per thread; 274 rows of 0.8 MB: 6.5 against 5.8.
    const int64_t unit = row_bytes % 16 == 0 ? 16 : (row_bytes % 4 == 0 ? 4 : 2);
    int64_t gx = row_bytes / unit / 256;
    if (gx < 1) gx = 1;
    if (gx > 4096) gx = 4096;
    int64_t gy = max_rows / 4;
    if (gy > 1024) gy = 1024;
    if (gy < 1) gy = 1;
    const dim3 grid((unsigned)gx, (unsigned)gy);
    const char* s = static_cast<const char*>(src);
    char* d = static_cast<char*>(dst);
    if (row_bytes % 16 == 0)
        hipLaunchKernelGGL((k_gather_rows<u32x4>), grid, dim3(256), 0, st, s, row_ids, next_slots, counts, max_rows, d, row_bytes);
    else if (row_bytes % 4 == 0)
        hipLaunchKernelGGL((k_gather_rows<uint32_t>), grid, dim3(256), 0, st, s, row_ids, next_slots, counts, max_rows, d, row_bytes);
    else
        hipLaunchKernelGGL((k_gather_rows<uint16_t>), grid, dim3(256), 0, st, s, row_ids, next_slots, counts, max_rows, d, row_bytes);
}

// Up to three int32 arrays copied in one launch (a NULL destination is skipped).
__global__ void k_copy3_i32(const int32_t* __restrict__ s0, int32_t* __restrict__ d0,
                            const int32_t* __restrict__ s1, int32_t* __restrict__ d1,
                            const int32_t* __restrict__ s2, int32_t* __restrict__ d2, int count) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x) {
        if (d0) d0[i] = s0[i];
        if (d1) d1[i] = s1[i];
        if (d2) d2[i] = s2[i];
    }
}

void launch_copy3_i32(const int32_t* s0, int32_t* d0, const int32_t* s1, int32_t* d1, const int32_t* s2,
                      int32_t* d2, int count, hipStream_t st) {
    if (count <= 0 || (!d0 && !d1 && !d2)) return;
    int grid = (count + 255) / 256;
    if (grid > 256) grid = 256;
    hipLaunchKernelGGL(k_copy3_i32, dim3(grid), dim3(256), 0, st, s0, d0, s1, d1, s2, d2, count);
}

__global__ void k_fill_u32(uint32_t* __restrict__ dst, uint32_t value, int count) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x) dst[i] = value;
}

void launch_fill_u32(uint32_t* dst, uint32_t value, int count, hipStream_t st) {
    if (count <= 0) return;
    int grid = (count + 255) / 256;
    if (grid > 256) grid = 256;
    hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(256), 0, st, dst, value, count);
}

// Fast-memory set from a list of class ids (already validated on the host: distinct, in range).
__global__ void k_set_hot(const int32_t* __restrict__ ids, int k, int n, int32_t* __restrict__ hot_ids,
                          uint8_t* __restrict__ in_hot, Counts* __restrict__ counts) {
    // single block
    for (int i = threadIdx.x; i < n; i += blockDim.x) in_hot[i] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < k; i += blockDim.x) {
        const int j = ids[i];
        hot_ids[i] = j;
        in_hot[j] = 1;
    }
    if (threadIdx.x == 0) counts->hot_k = k;
}

void launch_set_hot(const int32_t* ids, int k, int n, int32_t* hot_ids, uint8_t* in_hot, Counts* counts,
                    hipStream_t st) {
    hipLaunchKernelGGL(k_set_hot, dim3(1), dim3(1024), 0, st, ids, k, n, hot_ids, in_hot, counts);
}

}  // namespace smtm
