// Grouped bf16 GEMM with two wavefront groups that alternate between matrix work and memory work
// ("ping-pong"), for the expert FFN on gfx950.  C[r, n] = sum_k A[r, k] W_e[n, k] (+ bias, GELU).
//
// Workgroup = 8 wavefronts = 2 groups of 4; every SIMD hosts one wavefront of each group.  The
// output tile is 128 x BN; inside a group the 4 wavefronts form a 2x2 grid of 64 x BN/2 sub-tiles.
// Both groups cover the WHOLE tile but split each 64-deep k-step between them: group 0 multiplies
// k = 0..31 of the step, group 1 k = 32..63.  At the end the two partial sums are exchanged through
// LDS (each group finalises one 32-row half of every sub-tile), so the result is the fixed-order sum
// (group 0 part) + (group 1 part) and is reproducible.
//
// Schedule (one workgroup barrier per k-step; stage = LDS buffer of one k-step, 3 buffers):
//     group 0:  MFMAs(step t)                 | barrier t | issue DMA(step t+3) ; read fragments(step t+1)
//     group 1:  read fragments(step t)        | barrier t | issue DMA(step t+3) ; MFMAs(step t)
// so between two barriers one wavefront of each SIMD feeds the matrix pipe while the other one reads
// LDS, and they swap roles half a step later.  Barrier t publishes step t+1's tiles (every wavefront
// first waits for its own DMA of that step) and frees step t's buffer (all fragment reads of step t
// have completed before it), which the DMA for step t+3 then overwrites.
//
// Global -> LDS goes through global_load_lds_dwordx4 with 128-byte tile rows (a full cache line
// per row and DMA lane group), XOR-swizzled on 16-byte chunks; see ffn_mfma.hpp for the layout and
// the MFMA operand mapping.
#pragma once
#include "ffn_mfma.hpp"

namespace dicemoe {

// s_waitcnt lgkmcnt(0) only
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// blockIdx -> position in the tile sequence.  Workgroups go to the 8 XCDs round robin; hand every
// XCD patches of 32 consecutive positions (one per compute unit), so that the workgroups that run
// together on one XCD share A row tiles and W row tiles in its L2.
__device__ __forceinline__ int xcd_patch_position(int bid) {
    const int xcd = bid & 7, slot = bid >> 3;
    return (((slot >> 5) * 8 + xcd) << 5) + (slot & 31);
}

template <int BN, int GROUP_M, bool GELU, int DIAG = 0>
__global__ __launch_bounds__(512, 2) void ffn_gemm_bf16_pingpong_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const float* __restrict__ bias,
    bf16_t* __restrict__ C, int N, int K, const int32_t* __restrict__ seg_offsets,
    const int32_t* __restrict__ seg_expert, int n_seg, int n_tiles_n, int m_tiles_max)
{
    constexpr int BM = 128, BK = 64, STAGES = 3, NW = 8;
    constexpr int CH = 8;                        // 16-byte chunks per 128-byte tile row
    constexpr int RPI = 8;                       // tile rows per wave-wide DMA
    constexpr int WN = BN / 2;                   // sub-tile of a wavefront: 64 x WN
    constexpr int TN = WN / 32;
    constexpr int N_INST = (BM + BN) / RPI;
    static_assert(N_INST % NW == 0 && WN % 32 == 0, "tile shape");
    constexpr int QW = N_INST / NW;
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    static_assert(NW * TN * 4096 <= STAGES * STAGE_BYTES, "exchange buffer must fit in the stage buffers");
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // ---- which tile: bands of GROUP_M row tiles, row tile index fastest inside a band
    const int t = xcd_patch_position(blockIdx.x);
    const int band = t / (GROUP_M * n_tiles_n);
    const int in_band = t % (GROUP_M * n_tiles_n);
    const int left = m_tiles_max - band * GROUP_M;
    const int rows_here = left < GROUP_M ? left : GROUP_M;
    if (rows_here <= 0) return;
    const int tile_m = band * GROUP_M + in_band % rows_here;
    const int tile_n = in_band / rows_here;
    if (tile_n >= n_tiles_n) return;
    int seg, row0, row_end;
    if (!find_row_tile(seg_offsets, n_seg, BM, tile_m, seg, row0, row_end)) return;
    const int e = seg_expert[seg];
    const int n0 = tile_n * BN;
    const bf16_t* We = W + static_cast<size_t>(e) * N * K;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = wave >> 2;                   // 0: k 0..31 of every step, 1: k 32..63
    const int wm = (wave >> 1) & 1, wn = wave & 1;

    // ---- DMA sources (see ffn_mfma.hpp): instruction q fills combined rows q*8 .. q*8+7
    const bf16_t* src[QW];
#pragma unroll
    for (int i = 0; i < QW; ++i) {
        const int q = wave + i * NW;
        const int cr = q * RPI + lane / CH;
        const int slot = lane % CH;
        if (q * RPI < BM) {
            const int chunk = slot ^ chunk_swizzle<CH>(cr);
            int r = row0 + cr;
            if (r >= row_end) r = row_end - 1;
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

    // ---- fragment offsets inside a stage for this group's two k-slices (kk = 2*grp, 2*grp+1).
    // The swizzle only looks at the low four row bits, so the 32-row blocks of a sub-tile sit at
    // constant distances (32 rows * 128 bytes) and the second k-slice is the first one XOR 32 bytes.
    int a_base, b_base;
    {
        const int chunk = (2 * grp) * 2 + (lane >> 5);
        const int ra = wm * 64 + (lane & 31);
        const int rb = wn * WN + (lane & 31);
        a_base = (ra * CH + (chunk ^ chunk_swizzle<CH>(ra))) * 16;
        b_base = BM * BK * 2 + (rb * CH + (chunk ^ chunk_swizzle<CH>(rb))) * 16;
    }

    f32x16_v acc[2][TN];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    bf16x8_v af[2][2], bfr[2][TN];
    auto read_fragments = [&](int stage) {
        const char* st = smem + stage * STAGE_BYTES;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const char* pa = st + (a_base ^ (h * 32));
            const char* pb = st + (b_base ^ (h * 32));
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const u32x4_v v = *reinterpret_cast<const u32x4_v*>(pa + i * 4096);
                af[h][i] = *reinterpret_cast<const bf16x8_v*>(&v);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const u32x4_v v = *reinterpret_cast<const u32x4_v*>(pb + j * 4096);
                bfr[h][j] = *reinterpret_cast<const bf16x8_v*>(&v);
            }
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[h][i], bfr[h][j], acc[i][j], 0, 0, 0);
    };

    const int nk = K / BK;
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
        if (s < nk) issue_stage(s, s);
    // step 0 has landed once only the younger steps' loads (at most two) are outstanding
    if (nk >= 3) wait_vmcnt<2 * QW>();
    else if (nk == 2) wait_vmcnt<QW>();
    else wait_vmcnt<0>();
    block_barrier();

    // barrier kt: publishes step kt+1 (every wavefront has waited for its own DMA of that step; the
    // only younger loads are step kt+2's) and frees step kt's buffer for the DMA of step kt+3
    auto sync_and_refill = [&](int kt, int stage) {
        if (DIAG & 2) { if (kt == 0) wait_vmcnt<0>(); block_barrier(); return; }   // timing study: no refill
        if (kt + 2 < nk) wait_vmcnt<QW>();
        else wait_vmcnt<0>();
        block_barrier();
        if (kt + STAGES < nk) issue_stage(stage, kt + STAGES);
    };

    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (!(DIAG & 4) || kt == 0) read_fragments((DIAG & 2) ? 0 : stage);   // group 0: after barrier kt-1; group 1: before barrier kt
        if (grp == 1) {
            wait_lgkm0();                        // reads complete before the buffer is handed back
            sync_and_refill(kt, stage);
        }
        multiply();
        if (grp == 0) sync_and_refill(kt, stage);
        stage = (stage + 1 == STAGES) ? 0 : stage + 1;
    }

    // ---- exchange partial sums: group 0 finalises rows 0..31 of each 64-row sub-tile (i = 0),
    // group 1 rows 32..63 (i = 1).  Each wavefront parks the half it gives away in its own 4*TN KiB
    // region as [j][v/4][lane] 16-byte items, then adds the partner's parked half to the half it keeps.
    block_barrier();                             // every fragment read is done: stage buffers are free
    char* mine = smem + wave * (TN * 4096);
    const char* theirs = smem + (wave ^ 4) * (TN * 4096);
    auto park = [&](const f32x16_v(&half)[TN]) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4_v v = {half[j][4 * g], half[j][4 * g + 1], half[j][4 * g + 2], half[j][4 * g + 3]};
                *reinterpret_cast<f32x4_v*>(mine + (j * 4 + g) * 1024 + lane * 16) = v;
            }
    };
    auto absorb_and_store = [&](const f32x16_v(&half)[TN], int i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * WN + j * 32 + (lane & 31);
            const float bv = (bias && n < N) ? bias[static_cast<size_t>(e) * N + n] : 0.f;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4_v v = *reinterpret_cast<const f32x4_v*>(theirs + (j * 4 + g) * 1024 + lane * 16);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = row0 + wm * 64 + i * 32 + g * 8 + (lane >> 5) * 4 + u;
                    if (r < row_end && n < N && (!(DIAG & 1) || v[u] == 123456.789f)) {
                        float val = half[j][4 * g + u] + v[u] + bv;
                        if (GELU) val = gelu_erf(val);
                        C[static_cast<size_t>(r) * N + n] = float_to_bf16(val);
                    }
                }
            }
        }
    };
    if (grp == 0) park(acc[1]); else park(acc[0]);
    __syncthreads();
    if (grp == 0) absorb_and_store(acc[0], 0); else absorb_and_store(acc[1], 1);
}

template <int BN, int GROUP_M, bool GELU, int DIAG = 0>
static hipError_t launch_gemm_bf16_pingpong(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                            const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg,
                                            int max_rows, hipStream_t stream)
{
    auto kern = ffn_gemm_bf16_pingpong_kernel<BN, GROUP_M, GELU, DIAG>;
    constexpr int smem = 3 * (128 + BN) * 64 * 2;
    static bool configured = false;
    if (!configured) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (err != hipSuccess) return err;
        configured = true;
    }
    const int n_tiles_n = (N + BN - 1) / BN;
    const int m_tiles = (max_rows + 127) / 128 + n_seg;
    const int bands = (m_tiles + GROUP_M - 1) / GROUP_M;
    unsigned grid = static_cast<unsigned>(bands) * GROUP_M * n_tiles_n;
    grid = (grid + 255u) / 256u * 256u;          // whole patches for every XCD
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, stream, static_cast<const bf16_t*>(A),
                       static_cast<const bf16_t*>(W), bias, static_cast<bf16_t*>(C), N, K, seg_offsets, seg_expert,
                       n_seg, n_tiles_n, m_tiles);
    return hipGetLastError();
}

}  // namespace dicemoe
