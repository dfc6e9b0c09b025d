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
#include "ffn_wide.hpp"
#include "kernels.hpp"

namespace dicemoe {

// Register-staged kernel: A and W tiles of depth 64 go global -> registers -> LDS (one LDS buffer, the
// next tile's global loads are in flight during the MFMAs), so a workgroup needs only (BM+BN)*128
// bytes of LDS and two or three workgroups share a compute unit and hide each other's barriers,
// LDS stores and epilogues.
template <int BM, int BN, int OCC, bool XCD, bool GELU>
__global__ __launch_bounds__(256, OCC) void ffn_gemm_bf16_kernel(const bf16_t* __restrict__ A,
                                                                 const bf16_t* __restrict__ W,
                                                                 const float* __restrict__ bias,
                                                                 bf16_t* __restrict__ C, int N, int K,
                                                                 const int32_t* __restrict__ seg_offsets,
                                                                 const int32_t* __restrict__ seg_expert, int n_seg,
                                                                 int n_tiles_n, int m_tiles_max,
                                                                 const int32_t* __restrict__ row_index, int row_div,
                                                                 const int32_t* __restrict__ out_index,
                                                                 int32_t* __restrict__ status, int max_rows)
{
    constexpr int BK = 64;
    report_row_overflow(status, seg_offsets, n_seg, max_rows);
    constexpr int CH = BK / 8;          // 16-byte chunks per tile row
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_PASSES = BM / 32;   // 256 threads cover 32 rows x 8 chunks per pass
    constexpr int B_PASSES = BN / 32;
    constexpr int REGION = epilogue_region_bytes<TN>();
    static_assert(4 * REGION <= (BM + BN) * BK * 2, "epilogue slabs must fit in the tile buffer");
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

    // bias of this wavefront's columns, fetched now and used in the epilogue
    const int col_first = n0 + wn * WN;
    float bias_reg[(WN + 63) / 64];
    load_bias_columns<WN>(bias ? bias + static_cast<size_t>(e) * N + col_first : nullptr, N - col_first, lane, bias_reg);

    // global -> register staging: thread covers chunk (tid % 8) of rows (tid / 8) + 32*pass
    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;
    const u32x4_v* a_src[A_PASSES];
    const u32x4_v* b_src[B_PASSES];
#pragma unroll
    for (int p = 0; p < A_PASSES; ++p) {
        int r = row0 + ld_row + 32 * p;
        if (r >= row_end) r = row_end - 1;                    // clamp: tail rows repeat the last row
        if (row_index) r = row_index[r] / row_div;            // gather folded into the operand load
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

    // epilogue: the tile buffer is free (barrier above); every wavefront uses its own slab region
    char* region = lds + wave * REGION;
    float* bias_lds = reinterpret_cast<float*>(region + slab_bytes<TN>());
    stage_bias<WN>(bias_reg, bias_lds, lane);
    float4 bias_groups[TN][4];
    read_bias_groups<TN>(bias_lds, lane, bias_groups);
#pragma unroll
    for (int i = 0; i < TM; ++i)
        store_slab<TN, GELU>(acc[i], region, bias_groups, C, N, row0 + wm * WM + i * 32, row_end, col_first, lane,
                             out_index);
}

// float path (small workloads): 64x64 tile, depth 16, each thread a 4x4 block, plain FMAs in a
// fixed order.
template <bool GELU>
__global__ __launch_bounds__(256) void ffn_gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                           const float* __restrict__ bias, float* __restrict__ C,
                                                           int N, int K, const int32_t* __restrict__ seg_offsets,
                                                           const int32_t* __restrict__ seg_expert, int n_seg,
                                                           int n_tiles_n, const int32_t* __restrict__ row_index,
                                                           int row_div, const int32_t* __restrict__ out_index,
                                                           int32_t* __restrict__ status, int max_rows)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    report_row_overflow(status, seg_offsets, n_seg, max_rows);
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
    if (row_index) ar = row_index[ar] / row_div;
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
        const int r_out = out_index ? out_index[r] : r;      // scatter: the row out_index names
        if (r_out < 0) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float val = acc[i][j] + (bias ? bias[static_cast<size_t>(e) * N + n] : 0.f);
            if (GELU) val = gelu_erf(val);
            C[static_cast<size_t>(r_out) * N + n] = val;
        }
    }
}

// Second pass of a split reduction: C[r] = bf16(bias + partial[0][r] + partial[1][r] + ...), shares added in
// index order (no atomics: the same bits in every run).  One workgroup per 4 rows of a segment.
constexpr int kReduceRows = 4;
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int k_splits,
                                                           int partial_rows, const float* __restrict__ bias,
                                                           bf16_t* __restrict__ C, int N,
                                                           const int32_t* __restrict__ seg_offsets,
                                                           const int32_t* __restrict__ seg_expert, int n_seg,
                                                           const int32_t* __restrict__ out_index)
{
    int seg, row0, row_end;
    if (!find_row_tile(seg_offsets, n_seg, kReduceRows, blockIdx.x, seg, row0, row_end)) return;
    const int e = seg_expert[seg];
    const int groups = N / 8;                                   // 8 columns = 16 bytes of output per thread and turn
    const int rows = (row_end - row0) < kReduceRows ? (row_end - row0) : kReduceRows;
    const size_t share = static_cast<size_t>(partial_rows) * N;
    for (int c = threadIdx.x; c < rows * groups; c += blockDim.x) {
        const int r = row0 + c / groups;
        const int n = (c % groups) * 8;
        if (r >= partial_rows) continue;
        float v[8];
        if (bias) {
            const f32x4_v b0 = *reinterpret_cast<const f32x4_v*>(bias + static_cast<size_t>(e) * N + n);
            const f32x4_v b1 = *reinterpret_cast<const f32x4_v*>(bias + static_cast<size_t>(e) * N + n + 4);
#pragma unroll
            for (int t = 0; t < 4; ++t) { v[t] = b0[t]; v[4 + t] = b1[t]; }
        } else {
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = 0.f;
        }
        // the sum of the shares first, the bias last: the order of the unsplit kernel's epilogue
        float acc[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = 0.f;
        for (int sidx = 0; sidx < k_splits; ++sidx) {
            const float* p = partial + sidx * share + static_cast<size_t>(r) * N + n;
            const f32x4_v a0 = *reinterpret_cast<const f32x4_v*>(p);
            const f32x4_v a1 = *reinterpret_cast<const f32x4_v*>(p + 4);
#pragma unroll
            for (int t = 0; t < 4; ++t) { acc[t] += a0[t]; acc[4 + t] += a1[t]; }
        }
        const int dst = out_index ? out_index[r] : r;
        if (dst < 0) continue;
        u32x4_v packed;
#pragma unroll
        for (int t = 0; t < 4; ++t) packed[t] = pack_bf16x2(acc[2 * t] + v[2 * t], acc[2 * t + 1] + v[2 * t + 1]);
        *reinterpret_cast<u32x4_v*>(C + static_cast<size_t>(dst) * N + n) = packed;
    }
}

// max_rows == 0: no GEMM is launched, but the caller's bound is still checked against the table
__global__ void row_overflow_check_kernel(int32_t* __restrict__ status, const int32_t* __restrict__ seg_offsets, int n_seg)
{
    report_row_overflow(status, seg_offsets, n_seg, 0);
}

static hipError_t launch_row_overflow_check(int32_t* status, const int32_t* seg_offsets, int n_seg, hipStream_t stream)
{
    if (status == nullptr) return hipSuccess;
    hipLaunchKernelGGL(row_overflow_check_kernel, dim3(1), dim3(64), 0, stream, status, seg_offsets, n_seg);
    return hipGetLastError();
}

template <int BM, int BN, int OCC, bool XCD, bool GELU>
static hipError_t launch_gemm_bf16(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                   const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg, int max_rows,
                                   hipStream_t stream, const int32_t* row_index = nullptr, int row_div = 1,
                                   const int32_t* out_index = nullptr, int32_t* status = nullptr)
{
    const int n_tiles_n = (N + BN - 1) / BN;
    const int m_tiles = (max_rows + BM - 1) / BM + n_seg;
    const int bands = (m_tiles + 7) / 8;
    hipLaunchKernelGGL((ffn_gemm_bf16_kernel<BM, BN, OCC, XCD, GELU>), dim3(static_cast<unsigned>(bands) * 8 * n_tiles_n),
                       dim3(256), 0, stream, static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(W), bias,
                       static_cast<bf16_t*>(C), N, K, seg_offsets, seg_expert, n_seg, n_tiles_n, m_tiles, row_index,
                       row_div, out_index, status, max_rows);
    return hipGetLastError();
}

template <bool GELU>
static hipError_t launch_gemm_f32(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                  const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg, int max_rows,
                                  hipStream_t stream, const int32_t* row_index = nullptr, int row_div = 1,
                                  const int32_t* out_index = nullptr, int32_t* status = nullptr)
{
    const int n_tiles_n = (N + 63) / 64;
    const int m_tiles = (max_rows + 63) / 64 + n_seg;
    hipLaunchKernelGGL((ffn_gemm_f32_kernel<GELU>), dim3(static_cast<unsigned>(m_tiles) * n_tiles_n), dim3(256), 0,
                       stream, static_cast<const float*>(A), static_cast<const float*>(W), bias,
                       static_cast<float*>(C), N, K, seg_offsets, seg_expert, n_seg, n_tiles_n, row_index, row_div,
                       out_index, status, max_rows);
    return hipGetLastError();
}

// Tile shape for one bf16 grouped GEMM.  The wide kernel fetches fewer bytes per flop and keeps the
// matrix pipe fed from hand-scheduled wavefronts, and wins as soon as its tiles fill most of the chip:
//   256 x 192, one workgroup of eight wavefronts (4 x 2, each a 64 x 96 block; two per SIMD cover each
//     other's waits, +1 % over four wavefronts of 128 x 96) per compute unit, two stages of activations
//     and four of weights (all 160 KB of LDS; three with short reductions): the GEMM with the plain
//     epilogue, when that grid covers most of the 256 compute units.
//     The weights stream from HBM exactly once, and a barrier waits for the slowest of a step's loads:
//     every weight stage more gives those loads another step of flight (DiT-MoE-XL shape, GEMM2, same
//     box: 98 us with two weight stages, 86 - 91 with three, 82 - 86 with four);
//   128 x 192, two stages (80 KB of LDS), two workgroups per compute unit: the GEMM whose epilogue
//     evaluates GELU (one workgroup's MFMAs cover the other's epilogue arithmetic), and GEMMs between
//     one and two 256-wide rounds;
//   128 x 192, three stages, one workgroup per compute unit: grids of a quarter to one workgroup per
//     compute unit (few refreshed rows, or narrow outputs).  Alone on a compute unit a workgroup has nobody to hide its load
//     latency, and the third stage gives every load two steps of flight instead of one
//     (57 us instead of 78 us for GEMM2 at 4096 rows of the DiT-MoE-XL widths).
// Tiny problems stay on the 128 x 128 kernel, three workgroups per compute unit.
template <bool GELU>
static hipError_t launch_gemm_bf16_auto(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                        const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg,
                                        int max_rows, hipStream_t stream, const int32_t* row_index = nullptr,
                                        int row_div = 1, const int32_t* out_index = nullptr, float* partial = nullptr,
                                        size_t partial_bytes = 0, int32_t* status = nullptr)
{
    constexpr int kComputeUnits = 256;
    // tiles dealt to the XCDs by expert (one L2 per XCD: an expert's weight slabs are then fetched by one
    // XCD) whenever the segment table fits the lanes of a wavefront; else bands of row tiles
    const int by_expert = n_seg <= 64 ? 1 : 0;
    // expected tiles: every segment ends in a partial row tile, half a tile on average
    auto tiles = [&](int bm, int bn) {
        const long long m_tiles = (static_cast<long long>(max_rows) + static_cast<long long>(n_seg) * bm / 2 + bm - 1) / bm;
        return m_tiles * ((N + bn - 1) / bn);
    };
    const bool fits_192 = (N + 191) / 192 * 192 * 8 <= N * 9;          // at most 1/8 of the columns computed in vain
    // Few rows and a long reduction (the second GEMM after a small refresh fraction or for a small batch):
    // the 128 x 192 tiles do not fill the chip and each walks all of K.  With two or three workgroups per
    // tile, each on a share of K (float partial sums in the workspace, added by a second pass in a fixed
    // order), more compute units stream the weights at once: 54 -> 47 us at 2048 rows of the DiT-MoE-XL
    // widths.  Not worth it once the tiles fill the chip by themselves (57 vs 66 us at 4096 rows), nor when a
    // share is left with fewer than sixteen steps (DiT-MoE-S widths, K = 1536, 4096 rows: 32 us split in
    // three, 23 in two, 20 unsplit on three-stage tiles): the second pass then costs more than the split saves.
    if (!GELU && partial && fits_192 && by_expert) {
        const long long t23 = tiles(128, 192);
        int splits = 1;
        for (int sp = 3; sp >= 2 && splits == 1; --sp)       // the deepest split whose shares still fill the chip at most once
            if (t23 * sp * 20 <= kComputeUnits * 21 && K / 64 / sp >= 16 &&
                static_cast<size_t>(sp) * max_rows * N * sizeof(float) <= partial_bytes)
                splits = sp;
        if (splits > 1) {
            hipError_t err = launch_gemm_bf16_wide<2, 3, 2, 3, 3, GELU>(A, W, nullptr, C, N, K, seg_offsets, seg_expert, n_seg,
                                                                       max_rows, stream, row_index, row_div, nullptr,
                                                                       by_expert, partial, splits, status);
            if (err != hipSuccess) return err;
            const int blocks = (max_rows + kReduceRows - 1) / kReduceRows + n_seg;
            hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, stream, partial, splits, max_rows, bias,
                               static_cast<bf16_t*>(C), N, seg_offsets, seg_expert, n_seg, out_index);
            return hipGetLastError();
        }
    }
    if (!GELU && fits_192 && tiles(256, 192) * 10 >= kComputeUnits * 6) {
        if (K >= 320)      // four weight stages (all 160 KB of LDS): three steps of flight for the cold weight stream
            return launch_gemm_bf16_wide<2, 3, 2, 2, 4, GELU, 4, 2>(A, W, bias, C, N, K, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index, row_div, out_index, by_expert, nullptr, 1, status);
        if (K >= 256)
            return launch_gemm_bf16_wide<2, 3, 2, 2, 3, GELU, 4, 2>(A, W, bias, C, N, K, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index, row_div, out_index, by_expert, nullptr, 1, status);
        return launch_gemm_bf16_wide<4, 3, 2, 2, 2, GELU>(A, W, bias, C, N, K, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index, row_div, out_index, by_expert, nullptr, 1, status);
    }
    if (fits_192 && K >= 256 && tiles(128, 192) <= kComputeUnits && tiles(128, 192) * 4 >= kComputeUnits)
        return launch_gemm_bf16_wide<2, 3, 2, 3, 3, GELU>(A, W, bias, C, N, K, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index, row_div, out_index, by_expert, nullptr, 1, status);
    if (fits_192 && tiles(128, 192) * 2 >= kComputeUnits)
        return launch_gemm_bf16_wide<2, 3, 2, 2, 2, GELU>(A, W, bias, C, N, K, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index, row_div, out_index, by_expert, nullptr, 1, status);
    return launch_gemm_bf16<128, 128, 3, true, GELU>(A, W, bias, C, N, K, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index,
                                                           row_div, out_index, status);
}

// Every instantiation of the wide kernel that launch_gemm_bf16_auto can pick needs its LDS limit
// raised once per device.
template <bool GELU>
static hipError_t configure_gemm_bf16_auto()
{
    hipError_t err = configure_gemm_bf16_wide<2, 3, 2, 3, 3, GELU>();
    if (err == hipSuccess) err = configure_gemm_bf16_wide<2, 3, 2, 2, 3, GELU, 4, 2>();
    if (err == hipSuccess) err = configure_gemm_bf16_wide<2, 3, 2, 2, 4, GELU, 4, 2>();
    if (err == hipSuccess) err = configure_gemm_bf16_wide<4, 3, 2, 2, 2, GELU>();
    if (err == hipSuccess) err = configure_gemm_bf16_wide<2, 3, 2, 2, 2, GELU>();
    return err;
}

hipError_t prepare_expert_ffn()
{
    hipError_t err = configure_gemm_bf16_auto<true>();
    if (err == hipSuccess) err = configure_gemm_bf16_auto<false>();
    return err;
}

hipError_t launch_expert_ffn(bool bf16, const void* x_rows, const int32_t* row_index, int row_div,
                             const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg, int max_rows, int d,
                             int F, const void* W1, const float* b1, const void* W2, const float* b2, void* h_packed,
                             const int32_t* out_index, void* hidden, void* partial, size_t partial_bytes,
                             int32_t* status, hipStream_t stream, hipEvent_t between)
{
    if (max_rows == 0) return launch_row_overflow_check(status, seg_offsets, n_seg, stream);
    hipError_t err;
    if (bf16) {
        err = launch_gemm_bf16_auto<true>(x_rows, W1, b1, hidden, F, d, seg_offsets, seg_expert, n_seg, max_rows, stream,
                                          row_index, row_div, nullptr, nullptr, 0, status);
        if (err != hipSuccess) return err;
        if (between != nullptr && (err = hipEventRecord(between, stream)) != hipSuccess) return err;
        return launch_gemm_bf16_auto<false>(hidden, W2, b2, h_packed, d, F, seg_offsets, seg_expert, n_seg, max_rows, stream,
                                            nullptr, 1, out_index, static_cast<float*>(partial), partial_bytes);
    }
    err = launch_gemm_f32<true>(x_rows, W1, b1, hidden, F, d, seg_offsets, seg_expert, n_seg, max_rows, stream, row_index,
                                row_div, nullptr, status);
    if (err != hipSuccess) return err;
    if (between != nullptr && (err = hipEventRecord(between, stream)) != hipSuccess) return err;
    return launch_gemm_f32<false>(hidden, W2, b2, h_packed, d, F, seg_offsets, seg_expert, n_seg, max_rows, stream, nullptr, 1,
                                  out_index);
}

}  // namespace dicemoe
