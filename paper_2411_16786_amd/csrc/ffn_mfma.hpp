// Pieces shared by the bf16 expert-FFN kernels on gfx950 matrix cores (C[r, n] = sum_k A[r, k] W_e[n, k]
// + bias, optional GELU; rows grouped in segments that each use one expert's weights): vector types,
// the GELU evaluation, wait-count helpers, the segment-table walk, the LDS chunk swizzle and the
// epilogue that transposes a wavefront's results through LDS into whole-line stores.
//
// LDS tile layout: row-major rows of 64 bf16 (8 chunks of 16 bytes); the chunk index is XOR-swizzled
// with row bits so that an MFMA fragment read (32 consecutive rows, same chunk) touches every bank once.
//
// MFMA: v_mfma_f32_32x32x16_bf16.  Lane l supplies A[row l%32][k = 8*(l/32) .. +7] and
// B[col l%32][same k]; accumulator element v of lane l is C[8*(v/4) + 4*(l/32) + v%4][l%32].
#pragma once
#include "common.hpp"

namespace dicemoe {

typedef __bf16 bf16x8_v __attribute__((ext_vector_type(8)));
typedef float f32x16_v __attribute__((ext_vector_type(16)));
typedef float f32x4_v __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_v __attribute__((ext_vector_type(4)));   // 16 bytes in four VGPRs

#define DICEMOE_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define DICEMOE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

__device__ __forceinline__ float gelu_erf(float u) {
    return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
}

// GELU for the bf16 path, u Phi(u) with Phi the standard normal distribution function (the erf form,
// not the tanh approximation), written as  gelu(u) = max(u, 0) - a Phi(-a),  a = |u|.
// log2 Phi(-a) is smooth and nearly quadratic, so a degree-6 polynomial in a (weighted minimax fit on
// [0, 6], coefficients from gelu_fit.py beside the package) followed by one exp2 reproduces a Phi(-a)
// to 6e-8 absolute; beyond a = 6 the term is below 1e-8 and a is clamped.  In float arithmetic the
// result is within 3e-7 of the exact GELU everywhere, four orders of magnitude under the bf16 rounding
// (2^-9 relative) that it receives next.  Cost: one transcendental (exp2) and nine plain operations; the
// epilogue of the first GEMM evaluates it 4608 times per row.
__device__ __forceinline__ float gelu_erf_fast(float u) {
    const float a = fminf(fabsf(u), 6.0f);
    float p = fmaf(0x1.159ab2p-15f, a, -0x1.934b26p-11f);
    p = fmaf(p, a, 0x1.08ca02p-7f);
    p = fmaf(p, a, -0x1.b58d52p-5f);
    p = fmaf(p, a, -0x1.d5c80ep-2f);
    p = fmaf(p, a, -0x1.26b528p+0f);
    p = fmaf(p, a, -0x1.ffff18p-1f);
    const float tail = __builtin_amdgcn_exp2f(p);            // Phi(-a)
    return fmaf(-a, tail, fmaxf(u, 0.0f));
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14; expcnt, lgkmcnt left open)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// workgroup barrier without the memory fence of __syncthreads (which would drain the DMA queue);
// the empty asm statements keep the compiler from moving LDS accesses across it
__device__ __forceinline__ void block_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Launch check on behalf of the caller: the grid of a grouped GEMM is sized from the host's bound
// max_rows, so a segment table that holds more rows than that leaves tiles uncomputed.  The first
// thread of the first workgroup records it: status[0] = rows in the table if they exceed the bound,
// else 0; status[1] = the bound.
__device__ __forceinline__ void report_row_overflow(int32_t* __restrict__ status, const int32_t* __restrict__ seg_offsets,
                                                    int n_seg, int max_rows)
{
    if (status != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        const int total = seg_offsets[n_seg];
        status[0] = total > max_rows ? total : 0;
        status[1] = max_rows;
    }
}

// Walk the segment table: which segment and which rows does row tile `tile` cover?
__device__ __forceinline__ bool find_row_tile(const int32_t* __restrict__ seg_offsets, int n_seg, int BM, int tile,
                                              int& seg, int& row0, int& row_end)
{
    int begin = seg_offsets[0];
    for (int g = 0; g < n_seg; ++g) {
        const int end = seg_offsets[g + 1];
        const int cnt = end - begin;
        const int nt = (cnt + BM - 1) / BM;
        if (tile < nt) {
            seg = g;
            row0 = begin + tile * BM;
            row_end = end;
            return true;
        }
        tile -= nt;
        begin = end;
    }
    return false;
}

// Tile of workgroup `block` when the tiles are dealt to the eight XCDs by expert.  Workgroups go to
// the XCDs round robin (XCD = block mod 8) and every XCD has an L2 of its own, so the tiles that share
// an expert's weights should run on one XCD: each XCD then reads about one eighth of the weights
// instead of the slabs of every expert its share of a row-band ordering happens to touch.
//   home XCD of segment g = seg_expert[g] mod 8; an XCD's own list = the tiles of its segments, in
//   segment order, inside a segment in bands of `group_m` row tiles (row tile fastest);
//   cap = ceil(total tiles / 8): an XCD keeps the first cap tiles of its list; what is beyond the
//   cap (a hot expert) forms the overflow list, in XCD order, and is taken, in XCD order, by the
//   XCDs whose own list is shorter than cap.  Every tile is assigned exactly once and no XCD gets
//   more than cap; the grid must hold at least 8 * cap workgroups.
__device__ __forceinline__ bool find_tile_by_expert(const int32_t* __restrict__ seg_offsets,
                                                    const int32_t* __restrict__ seg_expert, int n_seg, int BM,
                                                    int n_tiles_n, int group_m, int block, int& seg, int& row0,
                                                    int& row_end, int& tile_n, int& expert)
{
    // n_seg <= 64: lane g holds segment g (one vector load instead of a walk of dependent scalar loads);
    // the uniform loops below pick the entries out with readlane
    const int lane = threadIdx.x & 63;
    int my_begin = 0, my_end = 0, my_home = 8, my_expert = 0;
    if (lane < n_seg) {
        my_begin = seg_offsets[lane];
        my_end = seg_offsets[lane + 1];
        my_expert = seg_expert[lane];
        my_home = my_expert & 7;
    }
    const int my_nt = (my_end - my_begin + BM - 1) / BM;
    const int x = block & 7, s = block >> 3;
    int own[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) own[i] = 0;
    for (int g = 0; g < n_seg; ++g) {
        const int tiles = __builtin_amdgcn_readlane(my_nt, g) * n_tiles_n;
        const int home = __builtin_amdgcn_readlane(my_home, g);
#pragma unroll
        for (int i = 0; i < 8; ++i) own[i] += (home == i) ? tiles : 0;
    }
    int total = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) total += own[i];
    if (total == 0) return false;
    const int cap = (total + 7) >> 3;
    int own_x = 0, spare_before = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int kept = own[i] < cap ? own[i] : cap;
        if (i == x) own_x = own[i];
        if (i < x) spare_before += cap - kept;
    }
    const int kept_x = own_x < cap ? own_x : cap;
    int list = x, idx = s;
    if (s >= kept_x) {                               // a slot beyond this XCD's own tiles takes overflow
        const int o = s - kept_x;
        if (o >= cap - kept_x) return false;
        int pos = spare_before + o;
        list = -1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int over = own[i] > cap ? own[i] - cap : 0;
            if (list < 0) {
                if (pos < over) { list = i; idx = cap + pos; }
                else pos -= over;
            }
        }
        if (list < 0) return false;
    }
    for (int g = 0; g < n_seg; ++g) {
        if (__builtin_amdgcn_readlane(my_home, g) != list) continue;
        const int nt = __builtin_amdgcn_readlane(my_nt, g);
        const int tiles = nt * n_tiles_n;
        if (idx < tiles) {
            const int band = idx / (group_m * n_tiles_n), in_band = idx % (group_m * n_tiles_n);
            const int left = nt - band * group_m;
            const int rows_here = left < group_m ? left : group_m;
            const int tile_m = band * group_m + in_band % rows_here;
            tile_n = in_band / rows_here;
            seg = g;
            row0 = __builtin_amdgcn_readlane(my_begin, g) + tile_m * BM;
            row_end = __builtin_amdgcn_readlane(my_end, g);
            expert = __builtin_amdgcn_readlane(my_expert, g);      // (no second, dependent trip to memory for it)
            return true;
        }
        idx -= tiles;
    }
    return false;
}

// chunk swizzle for 128-byte rows (8 chunks): any 8 or 16 consecutive rows at one logical chunk fall
// on distinct 16-byte bank groups.
template <int CH> __device__ __forceinline__ int chunk_swizzle(int row);
template <> __device__ __forceinline__ int chunk_swizzle<8>(int row) {
    return ((row >> 1) & 3) | ((((row) & 1) ^ ((row >> 3) & 1)) << 2);
}

// Epilogue shared by the bf16 kernels ("C-shuffle").  The MFMAs are issued with the operands swapped
// (W fragment as the row operand, activation fragment as the column operand), so accumulator element v
// of lane l belongs to output row (l % 32) and output column 8*(v/4) + 4*(l/32) + v%4 of its 32x32
// block: four consecutive columns per group of four registers.  Each wavefront adds the bias, applies
// GELU, packs four bf16 (8 bytes) and parks one 32-row slab of its sub-tile in a private LDS region
// with a padded pitch; it then reads the slab back row-contiguously, 16 bytes per lane, and stores
// full 16-byte pieces (whole cache lines per row) to global memory.  Only rows are predicated.
//
// The bias of the wavefront's WN columns is fetched once, at kernel start, into WN/64 registers per
// lane (load_bias_columns), long before it is needed; stage_bias parks it in LDS behind the slab and
// the groups read their four values from there.  (Fetching it from global memory group by group put a
// full memory round trip in front of every group.)
template <int WN>
__device__ __forceinline__ void load_bias_columns(const float* __restrict__ bias_n, int n_valid, int lane,
                                                  float (&reg)[(WN + 63) / 64])
{
#pragma unroll
    for (int b = 0; b < (WN + 63) / 64; ++b) {
        const int col = b * 64 + lane;
        reg[b] = (bias_n != nullptr && col < WN && col < n_valid) ? bias_n[col] : 0.f;
    }
}

template <int WN>
__device__ __forceinline__ void stage_bias(const float (&reg)[(WN + 63) / 64], float* bias_lds, int lane)
{
#pragma unroll
    for (int b = 0; b < (WN + 63) / 64; ++b) {
        const int col = b * 64 + lane;
        if (col < WN) bias_lds[col] = reg[b];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int TN> constexpr int slab_bytes() { return 32 * (TN * 32 * 2 + 16); }
template <int TN> constexpr int epilogue_region_bytes() { return slab_bytes<TN>() + TN * 32 * 4; }

// the wavefront's bias values in the layout the groups use them: bb[j][g] = columns j*32 + 8g + 4h .. +3
template <int TN>
__device__ __forceinline__ void read_bias_groups(const float* bias_lds, int lane, float4 (&bb)[TN][4])
{
    const int h = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) bb[j][g] = *reinterpret_cast<const float4*>(bias_lds + j * 32 + 8 * g + 4 * h);
}

template <int TN, bool GELU>
__device__ __forceinline__ void store_slab(const f32x16_v (&half)[TN], char* region, const float4 (&bb)[TN][4],
                                           bf16_t* __restrict__ C, int N, int row_first, int row_end, int col_first,
                                           int lane, const int32_t* __restrict__ out_index)
{
    constexpr int WN = TN * 32;
    constexpr int PITCH = WN * 2 + 16;            // bytes; keeps 16-byte alignment, staggers banks
    constexpr int CPR = WN / 8;                   // 16-byte chunks per slab row
    constexpr int NP = 32 * CPR / 64;             // 16-byte pieces per lane (32 * CPR = 128 TN: a whole number of wavefronts)
    const int m_local = lane & 31, h = lane >> 5;
    // destination row of every piece this lane will store: the packed row itself, or (scatter) the row
    // that out_index names for it; fetched first so that the arithmetic below covers the load
    int dst_row[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int r = row_first + (lane + 64 * p) / CPR;
        dst_row[p] = r < row_end ? (out_index ? out_index[r] : r) : -1;
    }
    // phase 1: arithmetic and parking, no LDS read in between (nothing to wait for).  A lane holds four
    // consecutive columns per group (columns 8g + 4h .. + 3 of block j, h = lane / 32).  Two groups at a
    // time, the two half-wavefronts swap one register pair (v_permlane32_swap) so that every lane ends up
    // with eight consecutive columns: half the LDS writes, 16 bytes each, and the 16 lanes of a write
    // cycle cover all banks (with 8-byte writes two rows shared their banks).
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
            uint2 packed[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int g = 2 * gp + q;
                float v0 = half[j][4 * g] + bb[j][g].x, v1 = half[j][4 * g + 1] + bb[j][g].y;
                float v2 = half[j][4 * g + 2] + bb[j][g].z, v3 = half[j][4 * g + 3] + bb[j][g].w;
                if (GELU) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
                packed[q] = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
            }
            // lanes 0..31 keep group 2gp and receive its upper four columns from lanes 32..63, which in turn
            // receive group 2gp+1's lower four columns
            const auto sx = __builtin_amdgcn_permlane32_swap(packed[0].x, packed[1].x, false, false);
            const auto sy = __builtin_amdgcn_permlane32_swap(packed[0].y, packed[1].y, false, false);
            const int nl = j * 32 + 16 * gp + 8 * h;
            *reinterpret_cast<u32x4_v*>(region + m_local * PITCH + nl * 2) = u32x4_v{sx[0], sy[0], sx[1], sy[1]};
        }
    __builtin_amdgcn_wave_barrier();
    // phase 2: all row-contiguous pieces of the slab in one batch of LDS reads, then the stores
    u32x4_v piece[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int idx = lane + 64 * p;
        piece[p] = *reinterpret_cast<const u32x4_v*>(region + (idx / CPR) * PITCH + (idx % CPR) * 16);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int idx = lane + 64 * p;
        const int n = col_first + (idx % CPR) * 8;
        if (dst_row[p] >= 0 && n < N) *reinterpret_cast<u32x4_v*>(C + static_cast<size_t>(dst_row[p]) * N + n) = piece[p];
    }
    __builtin_amdgcn_wave_barrier();
}

// The same epilogue without the trip through LDS: after the register swap every lane holds 16 bytes of
// one output row, and stores them itself (a store instruction then touches 32 rows, 32 bytes each).
template <int TN, bool GELU>
__device__ __forceinline__ void store_slab_direct(const f32x16_v (&half)[TN], const float4 (&bb)[TN][4],
                                                  bf16_t* __restrict__ C, int N, int row_first, int row_end,
                                                  int col_first, int lane, const int32_t* __restrict__ out_index)
{
    const int m_local = lane & 31, h = lane >> 5;
    const int r = row_first + m_local;
    const int dst = r < row_end ? (out_index ? out_index[r] : r) : -1;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
            uint2 packed[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int g = 2 * gp + q;
                float v0 = half[j][4 * g] + bb[j][g].x, v1 = half[j][4 * g + 1] + bb[j][g].y;
                float v2 = half[j][4 * g + 2] + bb[j][g].z, v3 = half[j][4 * g + 3] + bb[j][g].w;
                if (GELU) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
                packed[q] = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
            }
            const auto sx = __builtin_amdgcn_permlane32_swap(packed[0].x, packed[1].x, false, false);
            const auto sy = __builtin_amdgcn_permlane32_swap(packed[0].y, packed[1].y, false, false);
            const int n = col_first + j * 32 + 16 * gp + 8 * h;
            if (dst >= 0 && n < N)
                *reinterpret_cast<u32x4_v*>(C + static_cast<size_t>(dst) * N + n) = u32x4_v{sx[0], sy[0], sx[1], sy[1]};
        }
}

}  // namespace dicemoe
