// Grouped expert FFN (Algorithm 1, "x_e <- expert(x_d)"; experts are feed-forward networks):
// for every segment of packed rows, h = W2_e . gelu(W1_e . x + b1_e) + b2_e with the exact erf
// GELU.  Two grouped GEMMs with "rows x K" activations and "N x K" weights, both K-contiguous:
//   GEMM1: hidden[r, f] = gelu(sum_c x[r, c] W1_e[f, c] + b1_e[f])   (rounded to the storage type)
//   GEMM2: h[r, c]      =       sum_f hidden[r, f] W2_e[c, f] + b2_e[c]
//
// Variable-M scheduling: segment sizes live on the device, so the grid is launched for the worst
// case (ceil(max_rows/BM) + n_segments row tiles) and each workgroup finds its (segment, row tile)
// by walking the segment table; surplus workgroups exit at once.  Row tiles never straddle two
// segments, tail rows are clamped on load and masked on store.
//
// bf16 path: 256 threads = 4 wavefronts in a 2x2 grid, each wavefront owns a (BM/2)x(BN/2) block
// of 32x32 MFMA tiles (v_mfma_f32_32x32x16_bf16, float accumulation).  A and B tiles of depth
// BK = 64 go global -> registers -> LDS with the next tile's global loads in flight during the
// MFMAs.  LDS rows are 128 bytes; the 16-byte chunk index is XOR-swizzled with row bits so that
// the fragment reads (32 consecutive rows, same chunk) and the tile stores spread over all banks.
#include "common.hpp"
#include "ffn_mfma.hpp"
#include "kernels.hpp"

namespace dicemoe {

// Epilogue shared by the bf16 kernels ("C-shuffle").  The MFMAs are issued with the operands swapped
// (W fragment as the row operand, activation fragment as the column operand), so accumulator element v
// of lane l belongs to output row (l % 32) and output column 8*(v/4) + 4*(l/32) + v%4 of its 32x32
// block: four consecutive columns per group of four registers.  Each wavefront adds the bias, applies
// GELU, packs four bf16 (8 bytes) and parks one 32-row slab of its sub-tile in a private LDS region
// with a padded pitch; it then reads the slab back row-contiguously, 16 bytes per lane, and stores
// full 16-byte pieces (whole cache lines per row) to global memory.  Only rows are predicated.
template <int TN, bool GELU>
__device__ __forceinline__ void store_slab(const f32x16_v (&half)[TN], char* region, const float* __restrict__ bias_n,
                                           bf16_t* __restrict__ C, int N, int row_first, int row_end, int col_first,
                                           int lane)
{
    constexpr int WN = TN * 32;
    constexpr int PITCH = WN * 2 + 16;            // bytes; keeps 16-byte alignment, staggers banks
    constexpr int CPR = WN / 8;                   // 16-byte chunks per slab row
    const int m_local = lane & 31, h = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = j * 32 + 8 * g + 4 * h;
            float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
            if (bias_n) {
                const float4 bb = *reinterpret_cast<const float4*>(bias_n + nl);
                b0 = bb.x; b1 = bb.y; b2 = bb.z; b3 = bb.w;
            }
            float v0 = half[j][4 * g] + b0, v1 = half[j][4 * g + 1] + b1;
            float v2 = half[j][4 * g + 2] + b2, v3 = half[j][4 * g + 3] + b3;
            if (GELU) { v0 = gelu_erf_fast(v0); v1 = gelu_erf_fast(v1); v2 = gelu_erf_fast(v2); v3 = gelu_erf_fast(v3); }
            uint2 packed = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
            *reinterpret_cast<uint2*>(region + m_local * PITCH + nl * 2) = packed;
        }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int p = 0; p < (32 * CPR + 63) / 64; ++p) {
        const int idx = lane + 64 * p;
        const int row = idx / CPR, chunk = idx % CPR;
        if (idx < 32 * CPR) {
            const u32x4_v v = *reinterpret_cast<const u32x4_v*>(region + row * PITCH + chunk * 16);
            const int r = row_first + row;
            const int n = col_first + chunk * 8;
            if (r < row_end && n < N) *reinterpret_cast<u32x4_v*>(C + static_cast<size_t>(r) * N + n) = v;
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Register-staged kernel: A and W tiles of depth 64 go global -> registers -> LDS (one LDS buffer, the
// next tile's global loads are in flight during the MFMAs), so a workgroup needs only (BM+BN)*128
// bytes of LDS and two or three workgroups share a compute unit and hide each other's barriers,
// LDS stores and epilogues.
template <int BM, int BN, int OCC, bool XCD, bool PF, bool GELU>
__global__ __launch_bounds__(256, OCC) void ffn_gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                 const bf16_t* __restrict__ W,
                                                                 const float* __restrict__ bias,
                                                                 bf16_t* __restrict__ C, int N, int K,
                                                                 const int32_t* __restrict__ seg_offsets,
                                                                 const int32_t* __restrict__ seg_expert, int n_seg,
                                                                 int n_tiles_n, int m_tiles_max)
{
    constexpr int BK = 64;
    constexpr int CH = BK / 8;          // 16-byte chunks per tile row
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_PASSES = BM / 32;   // 256 threads cover 32 rows x 8 chunks per pass
    constexpr int B_PASSES = BN / 32;
    constexpr int SLAB = 32 * (WN * 2 + 16);
    static_assert(4 * SLAB <= (BM + BN) * BK * 2, "epilogue slabs must fit in the tile buffer");
    __shared__ __attribute__((aligned(16))) char lds[(BM + BN) * BK * 2];
    u32x4_v* As = reinterpret_cast<u32x4_v*>(lds);
    u32x4_v* Bs = As + BM * CH;

    // Tile sequence: bands of 8 row tiles, row tile fastest, so neighbours in the sequence share W
    // row tiles and a band shares its A rows.  Workgroups are handed to the 8 XCDs round robin
    // (blockIdx % 8); giving XCD x the x-th contiguous eighth of the sequence keeps each XCD's L2
    // working on its own bands instead of every L2 fetching every tile.
    constexpr int GROUP_M = 8;
    const int t = XCD ? (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
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

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // global -> register staging: thread covers chunk (tid % 8) of rows (tid / 8) + 32*pass
    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;
    const u32x4_v* a_src[A_PASSES];
    const u32x4_v* b_src[B_PASSES];
#pragma unroll
    for (int p = 0; p < A_PASSES; ++p) {
        int r = row0 + ld_row + 32 * p;
        if (r >= row_end) r = row_end - 1;                    // clamp: tail rows repeat the last row
        a_src[p] = reinterpret_cast<const u32x4_v*>(A + static_cast<size_t>(r) * K) + ld_chunk;
    }
#pragma unroll
    for (int p = 0; p < B_PASSES; ++p) {
        int n = n0 + ld_row + 32 * p;
        if (n >= N) n = N - 1;
        b_src[p] = reinterpret_cast<const u32x4_v*>(We + static_cast<size_t>(n) * K) + ld_chunk;
    }
    u32x4_v a_reg[A_PASSES], b_reg[B_PASSES];
#pragma unroll
    for (int p = 0; p < A_PASSES; ++p) a_reg[p] = a_src[p][0];
#pragma unroll
    for (int p = 0; p < B_PASSES; ++p) b_reg[p] = b_src[p][0];
    const int st_off = ld_row * CH + (ld_chunk ^ chunk_swizzle<8>(ld_row));   // + 32 rows per pass: same swizzle

    // fragment read offsets: 32-row blocks sit 32*128 bytes apart, k-slices differ in chunk bits only
    int a_off[BK / 16], b_off[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
        const int chunk = kk * 2 + (lane >> 5);
        const int ra = wm * WM + (lane & 31), rb = wn * WN + (lane & 31);
        a_off[kk] = ra * CH + (chunk ^ chunk_swizzle<8>(ra));
        b_off[kk] = rb * CH + (chunk ^ chunk_swizzle<8>(rb));
    }

    f32x16_v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = K / BK;
    for (int kt = 0; kt < nk; ++kt) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) As[st_off + p * 32 * CH] = a_reg[p];
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) Bs[st_off + p * 32 * CH] = b_reg[p];
        __syncthreads();
        if (kt + 1 < nk) {
            const int koff = (kt + 1) * CH;
#pragma unroll
            for (int p = 0; p < A_PASSES; ++p) a_reg[p] = a_src[p][koff];
#pragma unroll
            for (int p = 0; p < B_PASSES; ++p) b_reg[p] = b_src[p][koff];
        }
        if (PF) {
            // all fragments of the step first (one exposed LDS latency per step instead of four),
            // then hand the buffer back, then the MFMAs: they overlap the next step's LDS stores
            bf16x8_v af[BK / 16][TM], bfr[BK / 16][TN];
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const u32x4_v v = As[a_off[kk] + i * 32 * CH];
                    af[kk][i] = *reinterpret_cast<const bf16x8_v*>(&v);
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const u32x4_v v = Bs[b_off[kk] + j * 32 * CH];
                    bfr[kk][j] = *reinterpret_cast<const bf16x8_v*>(&v);
                }
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk][j], af[kk][i], acc[i][j], 0, 0, 0);
        } else {
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                bf16x8_v af[TM], bfr[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const u32x4_v v = As[a_off[kk] + i * 32 * CH];
                    af[i] = *reinterpret_cast<const bf16x8_v*>(&v);
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const u32x4_v v = Bs[b_off[kk] + j * 32 * CH];
                    bfr[j] = *reinterpret_cast<const bf16x8_v*>(&v);
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)     // operands swapped: see store_slab
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        }
    }
    if (PF) __syncthreads();                     // the slabs below reuse the tile buffer

    // epilogue: the tile buffer is free (barrier above); every wavefront uses its own slab region
    char* region = lds + wave * SLAB;
    const int col_first = n0 + wn * WN;
    const float* bias_n = bias ? bias + static_cast<size_t>(e) * N + col_first : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i)
        store_slab<TN, GELU>(acc[i], region, bias_n, C, N, row0 + wm * WM + i * 32, row_end, col_first, lane);
}

// float path (small workloads): 64x64 tile, depth 16, each thread a 4x4 block, plain FMAs in a
// fixed order.
template <bool GELU>
__global__ __launch_bounds__(256) void ffn_gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                           const float* __restrict__ bias, float* __restrict__ C,
                                                           int N, int K, const int32_t* __restrict__ seg_offsets,
                                                           const int32_t* __restrict__ seg_expert, int n_seg,
                                                           int n_tiles_n)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int tile_m = blockIdx.x / n_tiles_n;
    const int tile_n = blockIdx.x % n_tiles_n;
    int seg, row0, row_end;
    if (!find_row_tile(seg_offsets, n_seg, BM, tile_m, seg, row0, row_end)) return;
    const int e = seg_expert[seg];
    const int n0 = tile_n * BN;
    const float* We = W + static_cast<size_t>(e) * N * K;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;       // 16 x 16 threads, 4 columns x 4 rows each
    const int ld_r = tid >> 2, ld_c = (tid & 3) * 4;  // 64 rows x 4 float4 per tile

    int ar = row0 + ld_r; if (ar >= row_end) ar = row_end - 1;
    int bn = n0 + ld_r;   if (bn >= N) bn = N - 1;
    const float* a_src = A + static_cast<size_t>(ar) * K + ld_c;
    const float* b_src = We + static_cast<size_t>(bn) * K + ld_c;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += BK) {
        const float4 av = *reinterpret_cast<const float4*>(a_src + k0);
        const float4 bv = *reinterpret_cast<const float4*>(b_src + k0);
        As[ld_c + 0][ld_r] = av.x; As[ld_c + 1][ld_r] = av.y; As[ld_c + 2][ld_r] = av.z; As[ld_c + 3][ld_r] = av.w;
        Bs[ld_c + 0][ld_r] = bv.x; Bs[ld_c + 1][ld_r] = bv.y; Bs[ld_c + 2][ld_r] = bv.z; Bs[ld_c + 3][ld_r] = bv.w;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = row0 + ty * 4 + i;
        if (r >= row_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float val = acc[i][j] + (bias ? bias[static_cast<size_t>(e) * N + n] : 0.f);
            if (GELU) val = gelu_erf(val);
            C[static_cast<size_t>(r) * N + n] = val;
        }
    }
}

template <int BM, int BN, int OCC, bool XCD, bool PF, bool GELU>
static hipError_t launch_gemm_bf16(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                   const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg, int max_rows,
                                   hipStream_t stream)
{
    const int n_tiles_n = (N + BN - 1) / BN;
    const int m_tiles = (max_rows + BM - 1) / BM + n_seg;
    const int bands = (m_tiles + 7) / 8;
    hipLaunchKernelGGL((ffn_gemm_bf16_kernel<BM, BN, OCC, XCD, PF, GELU>), dim3(static_cast<unsigned>(bands) * 8 * n_tiles_n),
                       dim3(256), 0, stream, static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(W), bias,
                       static_cast<bf16_t*>(C), N, K, seg_offsets, seg_expert, n_seg, n_tiles_n, m_tiles);
    return hipGetLastError();
}

template <bool GELU>
static hipError_t launch_gemm_f32(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                  const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg, int max_rows,
                                  hipStream_t stream)
{
    const int n_tiles_n = (N + 63) / 64;
    const int m_tiles = (max_rows + 63) / 64 + n_seg;
    hipLaunchKernelGGL((ffn_gemm_f32_kernel<GELU>), dim3(static_cast<unsigned>(m_tiles) * n_tiles_n), dim3(256), 0,
                       stream, static_cast<const float*>(A), static_cast<const float*>(W), bias,
                       static_cast<float*>(C), N, K, seg_offsets, seg_expert, n_seg, n_tiles_n);
    return hipGetLastError();
}

hipError_t launch_expert_ffn(bool bf16, const void* x_packed, const int32_t* seg_offsets,
                             const int32_t* seg_expert, int n_seg, int max_rows, int d, int F, const void* W1,
                             const float* b1, const void* W2, const float* b2, void* h_packed, void* hidden,
                             hipStream_t stream)
{
    if (max_rows == 0) return hipSuccess;
    hipError_t err;
    if (bf16) {
        err = launch_gemm_bf16<128, 128, 3, true, false, true>(x_packed, W1, b1, hidden, F, d, seg_offsets, seg_expert, n_seg,
                                               max_rows, stream);
        if (err != hipSuccess) return err;
        return launch_gemm_bf16<128, 128, 3, true, false, false>(hidden, W2, b2, h_packed, d, F, seg_offsets, seg_expert, n_seg,
                                                 max_rows, stream);
    }
    err = launch_gemm_f32<true>(x_packed, W1, b1, hidden, F, d, seg_offsets, seg_expert, n_seg, max_rows, stream);
    if (err != hipSuccess) return err;
    return launch_gemm_f32<false>(hidden, W2, b2, h_packed, d, F, seg_offsets, seg_expert, n_seg, max_rows, stream);
}

}  // namespace dicemoe
