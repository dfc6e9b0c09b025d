// Grouped bf16 GEMM for the expert FFN on gfx950 matrix cores: C[r, n] = sum_k A[r, k] W_e[n, k]
// (+ bias, optional GELU), rows grouped in segments that each use one expert's weights.
//
// Data path: global memory -> LDS directly (global_load_lds_dwordx4: each lane moves 16 bytes,
// a wavefront fills 1 KiB of consecutive LDS, no staging registers) through a ring of STAGES
// tile buffers of depth BK, one workgroup barrier per k-step:
//     wait (own loads of step kt landed) ; barrier ; issue loads of step kt+STAGES-1 ; MFMAs of step kt
// The barrier both publishes step kt's tiles and proves that every wavefront has finished reading
// the buffer that the new loads overwrite (it was consumed in step kt-1).
//
// LDS tile layout: row-major rows of BK bf16 (BK/8 chunks of 16 bytes); the chunk index is
// XOR-swizzled with row bits so that an MFMA fragment read (32 consecutive rows, same chunk)
// touches every bank once.  The swizzle is applied on the global side of the DMA (which lane
// fetches which chunk), because the LDS side of the DMA is fixed: lane l lands at base + 16*l.
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

// chunk swizzles: 128-byte rows (8 chunks) and 64-byte rows (4 chunks).  Both make any 8 or 16
// consecutive rows at one logical chunk fall on distinct 16-byte bank groups.
template <int CH> __device__ __forceinline__ int chunk_swizzle(int row);
template <> __device__ __forceinline__ int chunk_swizzle<8>(int row) {
    return ((row >> 1) & 3) | ((((row) & 1) ^ ((row >> 3) & 1)) << 2);
}
template <> __device__ __forceinline__ int chunk_swizzle<4>(int row) {
    return ((row >> 2) & 3) ^ (((row >> 1) & 1) << 1);
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
                                           int lane)
{
    constexpr int WN = TN * 32;
    constexpr int PITCH = WN * 2 + 16;            // bytes; keeps 16-byte alignment, staggers banks
    constexpr int CPR = WN / 8;                   // 16-byte chunks per slab row
    constexpr int NP = 32 * CPR / 64;             // 16-byte pieces per lane (32 * CPR = 128 TN: a whole number of wavefronts)
    const int m_local = lane & 31, h = lane >> 5;
    // phase 1: arithmetic and parking, no LDS read in between (nothing to wait for)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = j * 32 + 8 * g + 4 * h;
            float v0 = half[j][4 * g] + bb[j][g].x, v1 = half[j][4 * g + 1] + bb[j][g].y;
            float v2 = half[j][4 * g + 2] + bb[j][g].z, v3 = half[j][4 * g + 3] + bb[j][g].w;
            if (GELU) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
            uint2 packed = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
            *reinterpret_cast<uint2*>(region + m_local * PITCH + nl * 2) = packed;
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
        const int r = row_first + idx / CPR;
        const int n = col_first + (idx % CPR) * 8;
        if (r < row_end && n < N) *reinterpret_cast<u32x4_v*>(C + static_cast<size_t>(r) * N + n) = piece[p];
    }
    __builtin_amdgcn_wave_barrier();
}

// blockIdx -> tile index.  MAP 0: identity.  MAP 1: workgroups are handed to the 8 XCDs round
// robin, so give each XCD one contiguous eighth of the tile sequence (its L2 then sees
// neighbouring tiles, which share A rows or W rows).
template <int MAP>
__device__ __forceinline__ int tile_of_block(int bid, int nblocks) {
    if (MAP == 0) return bid;
    const int per = nblocks >> 3;            // the launcher rounds the grid up to a multiple of 8
    return (bid & 7) * per + (bid >> 3);
}

template <int BM, int BN, int BK, int STAGES, int WAVES_M, int WAVES_N, int MAP, int GROUP_M, int OCC, bool GELU>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, OCC) void ffn_gemm_bf16_dma_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const float* __restrict__ bias,
    bf16_t* __restrict__ C, int N, int K, const int32_t* __restrict__ seg_offsets,
    const int32_t* __restrict__ seg_expert, int n_seg, int n_tiles_n, int m_tiles_max)
{
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int CH = BK / 8;                 // 16-byte chunks per tile row
    constexpr int RPI = 64 / CH;               // tile rows filled by one wave-wide DMA (1 KiB)
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int N_INST = (BM + BN) / RPI;    // DMA instructions per stage
    static_assert(N_INST % NW == 0, "DMA instructions must divide evenly over the wavefronts");
    static_assert(BM % RPI == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    constexpr int QW = N_INST / NW;            // per wavefront
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // ---- which tile
    const int t = tile_of_block<MAP>(blockIdx.x, gridDim.x);
    int tile_m, tile_n;
    if (GROUP_M > 0) {
        // bands of GROUP_M row tiles; inside a band the row tile index runs fastest
        const int band = t / (GROUP_M * n_tiles_n);
        const int in_band = t % (GROUP_M * n_tiles_n);
        const int rows_here = (m_tiles_max - band * GROUP_M) < GROUP_M ? (m_tiles_max - band * GROUP_M) : GROUP_M;
        if (rows_here <= 0) return;
        tile_m = band * GROUP_M + in_band % rows_here;
        tile_n = in_band / rows_here;
    } else {
        tile_m = t / n_tiles_n;
        tile_n = t % n_tiles_n;
    }
    if (tile_m >= m_tiles_max || tile_n >= n_tiles_n) return;
    int seg, row0, row_end;
    if (!find_row_tile(seg_offsets, n_seg, BM, tile_m, seg, row0, row_end)) return;
    const int e = seg_expert[seg];
    const int n0 = tile_n * BN;
    const bf16_t* We = W + static_cast<size_t>(e) * N * K;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- DMA sources: instruction q of a stage fills combined rows q*RPI .. q*RPI+RPI-1, where
    // combined row cr < BM is A row cr and cr >= BM is W row cr - BM.  This wavefront issues
    // q = wave, wave + NW, ...; lane l fetches the chunk that belongs at LDS slot (row, l % CH).
    const bf16_t* src[QW];
#pragma unroll
    for (int i = 0; i < QW; ++i) {
        const int q = wave + i * NW;
        const int cr = q * RPI + lane / CH;
        const int slot = lane % CH;
        if (q * RPI < BM) {
            const int chunk = slot ^ chunk_swizzle<CH>(cr);
            int r = row0 + cr;
            if (r >= row_end) r = row_end - 1;            // tail rows repeat the last row
            src[i] = A + static_cast<size_t>(r) * K + chunk * 8;
        } else {
            const int br = cr - BM;
            const int chunk = slot ^ chunk_swizzle<CH>(br);
            int n = n0 + br;
            if (n >= N) n = N - 1;
            src[i] = We + static_cast<size_t>(n) * K + chunk * 8;
        }
    }
    auto issue_stage = [&](int stage, int kt) {
        char* base = smem + stage * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < QW; ++i) {
            const int q = wave + i * NW;
            __builtin_amdgcn_global_load_lds(DICEMOE_GLOBAL_PTR(src[i] + kt * BK), DICEMOE_LDS_PTR(base + q * 1024),
                                             16, 0, 0);
        }
    };

    // ---- fragment read offsets (bytes inside a stage) for kk = 0; kk advances the chunk by 2
    int a_off[TM][BK / 16], b_off[TN][BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        const int chunk = kk * 2 + (lane >> 5);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = wm * WM + i * 32 + (lane & 31);
            a_off[i][kk] = (r * CH + (chunk ^ chunk_swizzle<CH>(r))) * 16;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int r = wn * WN + j * 32 + (lane & 31);
            b_off[j][kk] = BM * BK * 2 + (r * CH + (chunk ^ chunk_swizzle<CH>(r))) * 16;
        }
    }

    f32x16_v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / BK;
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < nk) issue_stage(s, s);

    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
        // my loads of step kt have landed once at most the younger steps' loads are outstanding
        const int younger = (nk - 1 - kt) < (STAGES - 2) ? (nk - 1 - kt) : (STAGES - 2);
        if (STAGES >= 3 && younger >= 1) {
            if (STAGES >= 4 && younger >= 2) wait_vmcnt<2 * QW>();
            else wait_vmcnt<QW>();
        } else {
            wait_vmcnt<0>();
        }
        block_barrier();
        if (kt + STAGES - 1 < nk) {
            int s2 = stage + STAGES - 1;
            if (s2 >= STAGES) s2 -= STAGES;
            issue_stage(s2, kt + STAGES - 1);
        }
        const char* st = smem + stage * STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_v af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const u32x4_v v = *reinterpret_cast<const u32x4_v*>(st + a_off[i][kk]);
                af[i] = *reinterpret_cast<const bf16x8_v*>(&v);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const u32x4_v v = *reinterpret_cast<const u32x4_v*>(st + b_off[j][kk]);
                bfr[j] = *reinterpret_cast<const bf16x8_v*>(&v);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (STAGES == 2) block_barrier();      // two buffers: the next loads overwrite this one
        stage = (stage + 1 == STAGES) ? 0 : stage + 1;
    }

    // ---- epilogue
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + (lane & 31);
        if (n >= N) continue;
        const float bv = bias ? bias[static_cast<size_t>(e) * N + n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = row0 + wm * WM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (r < row_end) {
                    float val = acc[i][j][v] + bv;
                    if (GELU) val = gelu_erf(val);
                    C[static_cast<size_t>(r) * N + n] = float_to_bf16(val);
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int STAGES, int WAVES_M, int WAVES_N, int MAP, int GROUP_M, int OCC, bool GELU>
static hipError_t launch_gemm_bf16_dma(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                       const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg,
                                       int max_rows, hipStream_t stream)
{
    auto kern = ffn_gemm_bf16_dma_kernel<BM, BN, BK, STAGES, WAVES_M, WAVES_N, MAP, GROUP_M, OCC, GELU>;
    constexpr int smem = STAGES * (BM + BN) * BK * 2;
    static bool configured = false;
    if (!configured) {
        if (smem > 64 * 1024) {
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (err != hipSuccess) return err;
        }
        configured = true;
    }
    const int n_tiles_n = (N + BN - 1) / BN;
    const int m_tiles = (max_rows + BM - 1) / BM + n_seg;
    int m_tiles_grid = m_tiles;
    if (GROUP_M > 0) m_tiles_grid = (m_tiles + GROUP_M - 1) / GROUP_M * GROUP_M;
    unsigned grid = static_cast<unsigned>(m_tiles_grid) * n_tiles_n;
    grid = (grid + 7u) / 8u * 8u;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES_M * WAVES_N * 64), smem, stream, static_cast<const bf16_t*>(A),
                       static_cast<const bf16_t*>(W), bias, static_cast<bf16_t*>(C), N, K, seg_offsets, seg_expert,
                       n_seg, n_tiles_n, m_tiles);
    return hipGetLastError();
}

}  // namespace dicemoe
