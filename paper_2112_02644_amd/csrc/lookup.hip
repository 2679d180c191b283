// Lookup: cosine similarity of every live frame's semantic vector with every class centre
// (arXiv 2112.02644, Eq. 1), accumulation over exit points with weight 2^(l-1) (Eq. 3), and per
// memory tier the highest / second-highest accumulated similarity with the exit rule of Eq. 4.
//
// Two launches per exit point:
//   score    one block per tile of 32 live frames x 128 classes.  It reads the frames' fp32 semantic
//            vectors and the centres (a few MB, from L2), takes the length of the vectors from the same
//            loads, contracts on the matrix cores (fp16 operands, fp32 accumulation) or in fp32 vector
//            arithmetic, updates SA in its epilogue and leaves, per frame and tile, the best and second
//            best SA of each memory tier.
//   decide   merges a frame's per-tile partial results in tile order and applies the exit rule; either as
//            a kernel of its own or at the head of the compaction kernel (compact.hip).
#include "internal.h"
#include <type_traits>
#include "decide.h"

namespace smtm {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float x) {
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

__device__ __forceinline__ float inv_norm_of(float nrm2) {
    // 0 marks a vector with zero or non-finite length: its similarities are defined as 0.
    if (!(nrm2 > 0.f) || !(nrm2 < __builtin_inff())) return 0.f;
    return 1.0f / sqrtf(nrm2);
}

// One wavefront per class: 1/|SC_j| and the unit-normalised fp16 copy (n_pad classes x Cp channels, zero
// padded, in the operand order of chat_index).
__global__ __launch_bounds__(256) void k_centre_prepare(const float* __restrict__ centres, int n, int C,
                                                        float* __restrict__ cinv,
                                                        _Float16* __restrict__ chat, int Cp,
                                                        int row_lo, int row_hi) {
    const int lane = threadIdx.x & 63;
    const int j = row_lo + blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= row_hi) return;
    if (j >= n) {                                       // padding rows of the fp16 copy
        for (int c = lane; c < Cp; c += 64) chat[chat_index(j, c, Cp)] = (_Float16)0.f;
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
        chat[chat_index(j, c, Cp)] = (_Float16)x;
    }
}

void launch_centre_prepare(const float* centres, int n, int C, float* cinv, _Float16* chat, int Cp,
                           int row_lo, int row_hi, hipStream_t st) {
    const int rows = row_hi - row_lo;
    if (rows <= 0) return;
    hipLaunchKernelGGL(k_centre_prepare, dim3((rows + 3) / 4), dim3(256), 0, st, centres, n, C, cinv,
                       chat, Cp, row_lo, row_hi);
}

// ---------------------------------------------------------------------------------------------
// What the scoring kernels share.
//
// Length of a semantic vector without a pass of its own: the encode kernels leave the largest |SV| of
// every frame (as the bit pattern of a non-negative float, which orders like the value).  From it a power
// of two is taken that brings the largest component into [1, 4), every component is multiplied by it
// (exact), and the sum of squares of the scaled components is accumulated from the very loads that feed
// the contraction.  The scaled components fit fp16 whatever the magnitude of the feature maps was, and
// the sum of squares can neither overflow nor vanish.
struct RowScale {
    float scale;                                         // power of two, 0 for a dead row
    bool dead;                                           // zero or non-finite vector: every similarity is 0
};

__device__ __forceinline__ RowScale row_scale_of(uint32_t max_bits) {
    RowScale r;
    r.dead = max_bits == 0u || max_bits >= 0x7f800000u;
    int field = 254 - (int)(max_bits >> 23);             // exponent field of 2^(127 - e): max * scale in [1, 2)
    field = field < 1 ? 1 : (field > 253 ? 253 : field);
    r.scale = r.dead ? 0.f : __builtin_bit_cast(float, (uint32_t)field << 23);
    return r;
}

// Largest |SV| of the frame in live slot `slot` (an epilogue row): thread (row = tid/8, k = tid%8) looks at the
// entries 8k .. 8k+7 of the slot (the encode kernel filled the first `slots` of the kRowMaxSlots = 64) and the 8
// threads of the row combine.  Any slot below max_rows is readable.
__device__ __forceinline__ uint32_t row_max_bits(const uint32_t* __restrict__ rowmax, int slots, int slot) {
    const int k = threadIdx.x & 7;
    const u32x4* p = reinterpret_cast<const u32x4*>(rowmax + (int64_t)slot * kRowMaxSlots + 8 * k);
    const u32x4 lo = p[0], hi = p[1];
    uint32_t a = 0u;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t x = 8 * k + e < slots ? lo[e] : 0u, y = 8 * k + 4 + e < slots ? hi[e] : 0u;
        a = x > a ? x : a;
        a = y > a ? y : a;
    }
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)a, off, 64);
        a = o > a ? o : a;
    }
    return a;
}

constexpr int SC_M = kScoreTileRows;                     // live frames per block tile
constexpr int SC_N = kScoreTileCols;                     // classes per block tile
constexpr int SC_LD = SC_N + 4;                          // padded LDS row (floats)

// Epilogue of a 32 x 128 tile whose dot products (of the scaled semantic vectors with the centre rows) sit in
// LDS as `copies` partial sums.  Thread t owns frame t/8 of the tile and 16 consecutive classes.
//   s = dot * inv_len(frame) * col_scale;   SA = SA_old + weight * s   (Eq. 1, Eq. 3)
// then the best / second best SA of the thread's classes per tier, merged over the 8 threads of the frame.
// sa_old holds the thread's 16 old SA values and hotw the fast-memory mask bytes of its 16 classes (both fetched
// before the contraction; sa_old is ignored when a.first).
__device__ __forceinline__ void score_epilogue(const ScoreArgs& a, const float* red, int copies, float ss,
                                               bool dead, const float* cinv, u32x4 hotw, int m0, int n0, int n_live,
                                               int fid, const f32x4 (&sa_old)[4]) {
    const int tid = threadIdx.x;
    const int row = tid >> 3, cg = tid & 7;
    const int slot = m0 + row;
    const bool live = slot < n_live;
    const int cls0 = n0 + cg * 16;
    float inv = inv_norm_of(ss);
    if (dead) inv = 0.f;
    float v[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f32x4 acc = *reinterpret_cast<const f32x4*>(red + row * SC_LD + cg * 16 + 4 * q);
        for (int w = 1; w < copies; ++w)                 // fixed order: the result does not depend on scheduling
            acc += *reinterpret_cast<const f32x4*>(red + (w * SC_M + row) * SC_LD + cg * 16 + 4 * q);
        v[4 * q] = acc.x; v[4 * q + 1] = acc.y; v[4 * q + 2] = acc.z; v[4 * q + 3] = acc.w;
    }
    const float ninf = -__builtin_inff();
    Top2 hot = {ninf, -1, ninf}, all = {ninf, -1, ninf};
    float* sa_row = a.SA + (int64_t)fid * a.n;
    float sa_new[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int cls = cls0 + i;
        float s = v[i] * inv;
        if (cinv) s *= cinv[cls < a.n ? cls : a.n - 1];
        if (inv == 0.f || !(fabsf(s) < __builtin_inff())) s = 0.f;
        v[i] = s;
        const float old = a.first ? 0.f : sa_old[i >> 2][i & 3];
        sa_new[i] = old + a.weight * s;
        const bool in = cls < a.n;
        const bool h = ((hotw[i >> 2] >> (8 * (i & 3))) & 0xffu) != 0;
        top2_push(all, sa_new[i], cls, in);
        top2_push(hot, sa_new[i], cls, in && h);
    }
    if (live) {
        const bool vec = (a.n & 3) == 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int cls = cls0 + 4 * q;
            if (vec && cls + 3 < a.n) {
                *reinterpret_cast<f32x4*>(sa_row + cls) = f32x4{sa_new[4 * q], sa_new[4 * q + 1], sa_new[4 * q + 2], sa_new[4 * q + 3]};
                if (a.sims_out)
                    *reinterpret_cast<f32x4*>(a.sims_out + (int64_t)slot * a.n + cls) = f32x4{v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (cls + e < a.n) {
                        sa_row[cls + e] = sa_new[4 * q + e];
                        if (a.sims_out) a.sims_out[(int64_t)slot * a.n + cls + e] = v[4 * q + e];
                    }
            }
        }
    }
    // the 8 threads of a frame hold its classes in ascending order of cg; merge in a fixed butterfly
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {
        float v1 = __shfl_xor(all.v1, off, 64); int id1 = __shfl_xor(all.id1, off, 64);
        float v2 = __shfl_xor(all.v2, off, 64);
        top2_merge(all, v1, id1, v2);
        v1 = __shfl_xor(hot.v1, off, 64); id1 = __shfl_xor(hot.id1, off, 64);
        v2 = __shfl_xor(hot.v2, off, 64);
        top2_merge(hot, v1, id1, v2);
    }
    if (live && cg == 0) {
        float* p = a.part + (int64_t)blockIdx.x * SC_FIELDS * a.part_stride + slot;
        p[0] = hot.v1;
        p[a.part_stride] = __builtin_bit_cast(float, hot.id1);
        p[2 * (int64_t)a.part_stride] = hot.v2;
        p[3 * (int64_t)a.part_stride] = all.v1;
        p[4 * (int64_t)a.part_stride] = __builtin_bit_cast(float, all.id1);
        p[5 * (int64_t)a.part_stride] = all.v2;
    }
}

// Old SA values of the thread's 16 classes.  The buffer has slack behind its last row, and the frame id comes
// from a list that only holds ids of this or an earlier batch, so the loads need no bounds checks.
__device__ __forceinline__ void fetch_sa_old(const ScoreArgs& a, int fid, int n0, f32x4 (&sa_old)[4]) {
    const int cg = threadIdx.x & 7;
    const float* sa_row = a.SA + (int64_t)fid * a.n + n0 + cg * 16;
    if (a.first) {
#pragma unroll
        for (int q = 0; q < 4; ++q) sa_old[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    } else if ((a.n & 3) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) sa_old[q] = *reinterpret_cast<const f32x4*>(sa_row + 4 * q);
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) sa_old[q] = f32x4{sa_row[4 * q], sa_row[4 * q + 1], sa_row[4 * q + 2], sa_row[4 * q + 3]};
    }
}

// ---------------------------------------------------------------------------------------------
// MFMA scoring.  v_mfma_f32_32x32x16_f16: a lane holds A[row = lane%32][k = 8*(lane/32) .. +7] and the same of B
// by column; acc[e] is C[row = 8*(e/4) + 4*(lane/32) + e%4][col = lane%32].
//   B (centres) is stored in exactly that order (chat_index), so the operand of a step is one contiguous 1 KB
//     load per wavefront, straight from L2 into registers.
//   A (semantic vectors, fp32, rows picked through the live list) is read with loads in which 16 neighbouring
//     lanes cover 256 contiguous bytes of a row, scaled, squared into the row's length, rounded to fp16 and
//     passed through a small LDS tile that belongs to the wavefront alone, from which every lane takes its row.
// There is no block barrier inside the K loop.  SPLITK: the 4 wavefronts each take every fourth stage of 64
// channels and all 128 classes of the tile, and their partial tiles are added in LDS in wavefront order.
// Otherwise (fewer than 4 stages) each takes all stages and 32 of the classes.
constexpr int kLeanStages = 1;                          // contractions this short take the lean scoring variant
constexpr int A_LD = 64 + 8;                             // halves per row of a wavefront's A tile (144 B: 16-byte reads without bank conflicts)

template <int NJ>
struct StageRegs {
    f32x4 a[8];                                          // load u: row 4u + lane/16 of the tile, floats 4*(lane%16) .. +3 of the stage
    u32x4 b[NJ][4];                                      // [class sub-tile][step]
};

template <int NJ, typename OFF>
__device__ __forceinline__ void fetch_stage(StageRegs<NJ>& R, const float* sv, const OFF (&a_off)[8], const _Float16* b_lane,
                                            int64_t b_tile_stride, int stage) {
#pragma unroll
    for (int u = 0; u < 8; ++u) R.a[u] = *reinterpret_cast<const f32x4*>(sv + a_off[u] + 64 * stage);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int u = 0; u < 4; ++u)
            R.b[j][u] = *reinterpret_cast<const u32x4*>(b_lane + j * b_tile_stride + (int64_t)(4 * stage + u) * 512);
}

template <int NJ>
__device__ __forceinline__ void multiply_stage(const StageRegs<NJ>& R, const float (&scale)[8], float (&ss)[8],
                                               _Float16* a_tile, floatx16 (&acc)[NJ]) {
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const f32x4 x = R.a[u] * scale[u];
        ss[u] += (x.x * x.x + x.y * x.y) + (x.z * x.z + x.w * x.w);
        const half4_t hv = {(_Float16)x.x, (_Float16)x.y, (_Float16)x.z, (_Float16)x.w};
        *reinterpret_cast<half4_t*>(a_tile + (4 * u + (lane >> 4)) * A_LD + 4 * (lane & 15)) = hv;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const half8_t av = *reinterpret_cast<const half8_t*>(a_tile + (lane & 31) * A_LD + 16 * ks + 8 * (lane >> 5));
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, __builtin_bit_cast(half8_t, R.b[j][ks]), acc[j], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the tile is rewritten by the next stage
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The variant for few stages keeps its registers under 256 so that two blocks share a CU: with a short K loop a
// block is little more than its chain of dependent memory round trips, and only other blocks can fill those.
// LEAN (long batches of narrow vectors: a single stage, a thousand blocks) goes further: one stage in flight per
// wavefront, registers at 128, four blocks per CU.  Measured on 4096 frames x 1000 classes x 24 channels: 15.7
// against 18.2 us; from two stages on the two variants take the same time.
template <bool SPLITK, bool LEAN>
__global__ __launch_bounds__(256, SPLITK ? 1 : (LEAN ? 4 : 2)) void k_score_mfma(ScoreArgs a, const _Float16* __restrict__ chat, int Cp) {
    static_assert(!(SPLITK && LEAN), "the lean variant does not split K");
    constexpr int NJ = SPLITK ? 4 : 1;
    constexpr int COPIES = SPLITK ? 4 : 1;
    __shared__ __attribute__((aligned(16))) float red[COPIES * SC_M * SC_LD];
    __shared__ __attribute__((aligned(16))) _Float16 a_tiles[4][SC_M * A_LD];
    __shared__ float ss_part[4][SC_M];
    __shared__ uint32_t row_bits[SC_M];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * SC_M, n0 = blockIdx.x * SC_N;
    const int n_stage = Cp / 64;
    const int j0 = SPLITK ? 0 : wave;                    // first 32-class sub-tile of this wavefront
    const int s0 = SPLITK ? wave : 0, sstep = SPLITK ? 4 : 1;
    const int my_n = s0 < n_stage ? (n_stage - s0 + sstep - 1) / sstep : 0;
    auto stage_of = [&](int i) { return s0 + i * sstep; };

    // Semantic vectors and their maxima are stored by live slot, so everything the contraction needs is addressed
    // without the live list: live count, vectors, maxima, centre operands, fast-memory mask and the frame id of
    // the epilogue row (for SA, which is kept by frame) are all requested before any of them is waited for.  Rows
    // of slots past the live count are readable (the buffers hold max_rows rows) and never used.
    int n_live = a.counts->n_live;
    const int slot_e = m0 + (tid >> 3) < a.max_rows ? m0 + (tid >> 3) : a.max_rows - 1;
    int fid_e = a.frame_ids[slot_e];                     // frame of this thread's epilogue row
    const int64_t b_tile_stride = (int64_t)(Cp >> 4) * 512;              // halves between two 32-class tiles
    const _Float16* b_lane = chat + (int64_t)((n0 >> 5) + j0) * b_tile_stride + lane * 8;
    const u32x4 hotw = *reinterpret_cast<const u32x4*>(a.in_hot + n0 + (tid & 7) * 16);   // the mask is padded to whole tiles
    typedef typename std::conditional<LEAN, int32_t, int64_t>::type off_t;   // the lean launch checks that 32 bits hold the offsets
    off_t a_off[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int slot = m0 + 4 * u + (lane >> 4);
        a_off[u] = (off_t)(slot < a.max_rows ? slot : a.max_rows - 1) * a.ldv + 4 * (lane & 15);
    }
    const uint32_t bits_e = row_max_bits(a.rowmax, a.rowmax_slots, slot_e);
    StageRegs<NJ> R0;
    if (my_n > 0) fetch_stage(R0, a.sv, a_off, b_lane, b_tile_stride, stage_of(0));
    asm volatile("" : "+v"(fid_e), "+s"(n_live));
    if (n_live > a.max_rows) n_live = a.max_rows;
    if (m0 >= n_live) return;                            // uniform over the block

    f32x4 sa_old[4];
    fetch_sa_old(a, fid_e, n0, sa_old);
    if ((tid & 7) == 0) row_bits[tid >> 3] = bits_e;
    __syncthreads();
    float scale[8], ss[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { scale[u] = row_scale_of(row_bits[4 * u + (lane >> 4)]).scale; ss[u] = 0.f; }

    floatx16 acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    _Float16* a_tile = a_tiles[wave];
    if constexpr (LEAN) {
        for (int i = 0; i < my_n; ++i) {                 // other blocks on the CU cover the wait
            if (i > 0) fetch_stage(R0, a.sv, a_off, b_lane, b_tile_stride, stage_of(i));
            multiply_stage<NJ>(R0, scale, ss, a_tile, acc);
        }
    } else {
    StageRegs<NJ> R1;
    for (int i = 0; i < my_n; i += 2) {                  // two stages per trip so that the register sets are static:
        if (i + 1 < my_n) fetch_stage(R1, a.sv, a_off, b_lane, b_tile_stride, stage_of(i + 1));   // the next stage is
        multiply_stage<NJ>(R0, scale, ss, a_tile, acc);                                                // in flight while this
        if (i + 1 >= my_n) break;                                                                      // one is multiplied
        if (i + 2 < my_n) fetch_stage(R0, a.sv, a_off, b_lane, b_tile_stride, stage_of(i + 2));
        multiply_stage<NJ>(R1, scale, ss, a_tile, acc);
    }
    }

    // partial sums of squares (16 lanes share a row) and partial tiles to LDS
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        float t = ss[u];
        t += __shfl_xor(t, 1, 64); t += __shfl_xor(t, 2, 64); t += __shfl_xor(t, 4, 64); t += __shfl_xor(t, 8, 64);
        if ((lane & 15) == 0) ss_part[wave][4 * u + (lane >> 4)] = t;
    }
    float* my_red = red + (SPLITK ? wave * SC_M * SC_LD : 0);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = 8 * (e >> 2) + 4 * h + (e & 3);
            my_red[row * SC_LD + (j0 + j) * 32 + r] = acc[j][e];
        }
    __syncthreads();
    const int row_e = tid >> 3;
    float ss_row = ss_part[0][row_e];
    if (SPLITK) ss_row = ((ss_row + ss_part[1][row_e]) + ss_part[2][row_e]) + ss_part[3][row_e];
    const RowScale re = row_scale_of(bits_e);            // whether the epilogue row is dead
    score_epilogue(a, red, COPIES, ss_row, re.dead, nullptr, hotw, m0, n0, n_live, fid_e, sa_old);
}

void launch_score_mfma(const ScoreArgs& a, const _Float16* chat, int Cp, hipStream_t st) {
    // centres are padded to kRowPad = 128 classes and Cp is a multiple of 64: a tile never reads outside them
    dim3 grid((a.n + SC_N - 1) / SC_N, (a.max_rows + SC_M - 1) / SC_M);
    // Splitting K over the wavefronts shortens a block's chain of stages but costs the registers that would let
    // two blocks share a CU: worth it for long K, or when there are too few blocks to fill the CUs twice anyway.
    const int n_stage = Cp / 64;
    const bool split = n_stage >= 4 && (n_stage >= 16 || (int64_t)grid.x * grid.y <= 512);
    const bool lean = !split && n_stage <= kLeanStages && (int64_t)grid.x * grid.y > 512 &&
                      (int64_t)a.max_rows * a.ldv < (int64_t)1 << 31;
    if (split) hipLaunchKernelGGL((k_score_mfma<true, false>), grid, dim3(256), 0, st, a, chat, Cp);
    else if (lean) hipLaunchKernelGGL((k_score_mfma<false, true>), grid, dim3(256), 0, st, a, chat, Cp);
    else hipLaunchKernelGGL((k_score_mfma<false, false>), grid, dim3(256), 0, st, a, chat, Cp);
}

// ---------------------------------------------------------------------------------------------
// fp32 scoring (fp32 feature maps, or on request): same tile, same epilogue; the contraction runs in fp32
// vector arithmetic from LDS tiles of 16 channels.  Thread t owns frame t/8 and 16 consecutive classes, which
// is also how the epilogue wants them, so the accumulators only pass through LDS to share its code.
constexpr int FP_K = 16;

__global__ __launch_bounds__(256) void k_score_fp32(ScoreArgs a, const float* __restrict__ centres,
                                                    const float* __restrict__ cinv, int C) {
    __shared__ __attribute__((aligned(16))) float red[SC_M * SC_LD];
    __shared__ float As[FP_K][SC_M + 1];
    __shared__ __attribute__((aligned(16))) float Bs[FP_K][SC_N + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * SC_M, n0 = blockIdx.x * SC_N;
    const int row = tid >> 3, cg = tid & 7;
    int n_live = a.counts->n_live;
    const int slot_e = m0 + row < a.max_rows ? m0 + row : a.max_rows - 1;
    int fid = a.frame_ids[slot_e];
    asm volatile("" : "+v"(fid), "+s"(n_live));
    if (n_live > a.max_rows) n_live = a.max_rows;
    if (m0 >= n_live) return;                            // uniform over the block
    const RowScale rs = row_scale_of(row_max_bits(a.rowmax, a.rowmax_slots, slot_e));
    f32x4 sa_old[4];
    fetch_sa_old(a, fid, n0, sa_old);
    const u32x4 hotw = *reinterpret_cast<const u32x4*>(a.in_hot + n0 + cg * 16);          // the mask is padded to whole tiles
    // loaders: A tile 32 frames x 16 channels, two per thread (the 8 threads of a frame load its 16 channels);
    // B tile 128 classes x 16 channels, eight per thread
    const float* a_ptr = a.sv + (int64_t)slot_e * a.ldv + cg * 2;       // by live slot; padded with zeros up to ldv
    const int b_cls = n0 + (tid >> 1), b_k = (tid & 1) * 8;
    const float* b_ptr = b_cls < a.n ? centres + (int64_t)b_cls * C : nullptr;
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    float ss = 0.f;
    for (int k0 = 0; k0 < C; k0 += FP_K) {
        const float x0 = a_ptr[k0] * rs.scale, x1 = a_ptr[k0 + 1] * rs.scale;   // k0 + 1 < ldv: ldv is a multiple of 64
        ss += x0 * x0 + x1 * x1;
        As[cg * 2][row] = x0;
        As[cg * 2 + 1][row] = x1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = k0 + b_k + i;
            Bs[b_k + i][tid >> 1] = (b_ptr && k < C) ? b_ptr[k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FP_K; ++kk) {
            const float av = As[kk][row];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 b = *reinterpret_cast<const f32x4*>(&Bs[kk][cg * 16 + 4 * q]);
                acc[4 * q] += av * b.x; acc[4 * q + 1] += av * b.y; acc[4 * q + 2] += av * b.z; acc[4 * q + 3] += av * b.w;
            }
        }
        __syncthreads();
    }
    // sum of squares of the frame: its 8 loader threads are 8 neighbouring lanes
    ss += __shfl_xor(ss, 1, 64);
    ss += __shfl_xor(ss, 2, 64);
    ss += __shfl_xor(ss, 4, 64);
#pragma unroll
    for (int i = 0; i < 16; ++i) red[row * SC_LD + cg * 16 + i] = acc[i];
    __syncthreads();
    score_epilogue(a, red, 1, ss, rs.dead, cinv, hotw, m0, n0, n_live, fid, sa_old);
}

void launch_score_fp32(const ScoreArgs& a, const float* centres, const float* cinv, int C, hipStream_t st) {
    dim3 grid((a.n + SC_N - 1) / SC_N, (a.max_rows + SC_M - 1) / SC_M);
    hipLaunchKernelGGL(k_score_fp32, grid, dim3(256), 0, st, a, centres, cinv, C);
}

// ---------------------------------------------------------------------------------------------
// The decision as a kernel of its own (smtm_lookup); smtm_lookup_exit runs it at the head of the compaction.
__global__ __launch_bounds__(256) void k_decide(DecideArgs g) {
    int n_live = g.counts->n_live;
    if (n_live > g.max_rows) n_live = g.max_rows;
    for (int slot = blockIdx.x * 256 + threadIdx.x; slot < n_live; slot += gridDim.x * 256) decide_slot(g, slot);
}

void launch_decide(const DecideArgs& g, hipStream_t st) {
    int grid = (g.max_rows + 255) / 256;
    if (grid > 1024) grid = 1024;
    hipLaunchKernelGGL(k_decide, dim3(grid), dim3(256), 0, st, g);
}

// ---------------------------------------------------------------------------------------------
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

}  // namespace smtm
