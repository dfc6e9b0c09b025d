// Wide-tile grouped bf16 GEMM for the expert FFN (Algorithm 1, "x_e <- expert(x_d)"): one workgroup
// of four wavefronts per compute unit owns a (64 TM) x (64 TN) output tile, each wavefront a
// (32 TM) x (32 TN) block of 32x32 MFMA tiles, so that the bytes fetched per flop fall to
// (BM + BN) / (BM BN) -- half of what a 128 x 128 tile needs at 256 x 256 -- and the L2 -> LDS path
// stops being the limit.
//
// Data path: global -> LDS directly (16 bytes per lane, 1 KiB per wavefront instruction), two
// stages of depth 64.  The loop is scheduled by hand, one instruction per scheduling region:
// every MFMA is followed by at most one fragment read (for the next 16-deep slice, into the other
// fragment register set) and one direct-to-LDS load, so the matrix pipe never waits for the
// wavefront's own memory instructions to issue.  One workgroup barrier per 64-deep step, placed
// before the MFMAs of the last slice: at that point every wavefront has read all fragments of the
// current stage (so the stage can be refilled) and its own loads of the next stage have landed.
#pragma once
#include <type_traits>
#include "ffn_mfma.hpp"

namespace dicemoe {

template <int N>
__device__ __forceinline__ void wait_lgkmcnt() {
    __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | ((N & 0xF) << 8));
}

#define DICEMOE_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Build-time timing aid (off in the library build): bit 0 drops the epilogue, bit 1 the stage loads,
// bit 2 the fragment reads, bit 3 everything after the tile lookup.  Results are wrong with any bit set.
#ifndef DICEMOE_FFN_DIAG
#define DICEMOE_FFN_DIAG 0
#endif

// workgroups per compute unit that the LDS footprint allows (the register budget follows from it)
constexpr int wide_occupancy(int tm, int tn, int ast, int wst, int wgm, int wgn) {
    return (ast * tm * wgm + wst * tn * wgn) * 32 * 128 <= 80 * 1024 ? 2 : 1;
}

template <int TM, int TN, int SPREAD, int AST, int WST, bool GELU, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN, wide_occupancy(TM, TN, AST, WST, WGM, WGN)) void ffn_gemm_bf16_wide_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const float* __restrict__ bias,
    bf16_t* __restrict__ C, int N, int K, const int32_t* __restrict__ seg_offsets,
    const int32_t* __restrict__ seg_expert, int n_seg, int n_tiles_n, int m_tiles_max,
    const int32_t* __restrict__ row_index, int row_div, const int32_t* __restrict__ out_index, int by_expert,
    float* __restrict__ partial, int partial_rows, int32_t* __restrict__ status)
{
#if DICEMOE_FFN_DIAG
    constexpr int DIAG = DICEMOE_FFN_DIAG;
#endif
    constexpr int NW = WGM * WGN;                  // wavefronts, WGM along the rows by WGN along the columns
    constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
    constexpr int WM = 32 * TM, WN = 32 * TN;
    constexpr int CH = 8;                          // 16-byte chunks per 64-deep tile row
    constexpr int QA = BM / (8 * NW), QB = BN / (8 * NW);      // direct-to-LDS loads per wavefront and stage (8 rows each)
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "every wavefront loads whole groups of eight rows");
    constexpr int QW = QA + QB;
    constexpr int ABYTES = BM * 128, WBYTES = BN * 128;      // one stage of each operand
    constexpr int NFRAG = TM + TN;
    constexpr int NMFMA = TM * TN;
    constexpr int GROUP_M = 8;
    constexpr int REGION = epilogue_region_bytes<TN>();
    static_assert(NW * REGION <= AST * ABYTES + WST * WBYTES, "epilogue slabs must fit in the stage buffers");
    static_assert((AST == 2 && (WST == 2 || WST == 3 || WST == 4)) || (AST == 3 && WST == 3) || (AST == 4 && WST == 4),
                  "ring depths (A, W): (2,2), (2,3), (2,4), (3,3), (4,4)");
    static_assert(NMFMA >= NFRAG, "one fragment read per MFMA slot");
    static_assert(SPREAD >= 1 && SPREAD <= 4, "a refill is issued within the four slices before it is needed");
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    char* const a_lds = smem;
    char* const w_lds = smem + AST * ABYTES;

    // launch check for the caller: did the segment table hold more rows than the grid was sized for?
    report_row_overflow(status, seg_offsets, n_seg, partial_rows);
    // ---- which tile (bands of GROUP_M row tiles, XCD x takes the x-th eighth of the sequence)
    int seg, row0, row_end, tile_n, e = -1;
    if (by_expert) {
        if (!find_tile_by_expert(seg_offsets, seg_expert, n_seg, BM, n_tiles_n, GROUP_M, blockIdx.x, seg, row0, row_end,
                                 tile_n, e))
            return;
    } else {
        const int t = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
        const int band = t / (GROUP_M * n_tiles_n);
        const int in_band = t % (GROUP_M * n_tiles_n);
        const int left = m_tiles_max - band * GROUP_M;
        const int rows_here = left < GROUP_M ? left : GROUP_M;
        if (rows_here <= 0) return;
        const int tile_m = band * GROUP_M + in_band % rows_here;
        tile_n = in_band / rows_here;
        if (tile_n >= n_tiles_n) return;
        if (!find_row_tile(seg_offsets, n_seg, BM, tile_m, seg, row0, row_end)) return;
    }
#if DICEMOE_FFN_DIAG
    if (DIAG & 8) {                                 // timing aid: the tile lookup alone
        if (seg + row0 + row_end + tile_n == -12345) C[0] = 1;
        return;
    }
#endif
    if (!by_expert) e = seg_expert[seg];
    const int n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // bias of this wavefront's columns, fetched now and used in the epilogue
    const int col_first = n0 + wn * WN;
    float bias_reg[(WN + 63) / 64];
    load_bias_columns<WN>(bias ? bias + static_cast<size_t>(e) * N + col_first : nullptr, N - col_first, lane, bias_reg);

    // ---- direct-to-LDS sources.  Load q of an operand fills tile rows 8q .. 8q+7; lane l lands at
    // LDS slot (row 8q + l/8, l%8) and therefore fetches the chunk that the swizzle assigns to that slot.
    // With a row index, packed row r is read from A row row_index[r] / row_div (the pair id of
    // the packed row divided by k is its token): the dispatch gather folded into the operand load.
    const char* a_base = reinterpret_cast<const char*>(A);
    const char* w_base = reinterpret_cast<const char*>(W + (static_cast<size_t>(e) * N + n0) * K);
    uint32_t goff[QW];
#pragma unroll
    for (int i = 0; i < QA; ++i) {
        const int row = (wave * QA + i) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ chunk_swizzle<CH>(row);
        int r = row0 + row;
        if (r >= row_end) r = row_end - 1;                    // tail rows repeat the last row
        const uint32_t src = row_index ? static_cast<uint32_t>(row_index[r] / row_div) : static_cast<uint32_t>(r);
        goff[i] = src * static_cast<uint32_t>(K) * 2u + chunk * 16;     // the launcher checks that A spans < 4 GiB
    }
#pragma unroll
    for (int i = 0; i < QB; ++i) {
        const int row = (wave * QB + i) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ chunk_swizzle<CH>(row);
        int n = n0 + row;
        if (n >= N) n = N - 1;
        goff[QA + i] = static_cast<uint32_t>(n - n0) * static_cast<uint32_t>(K) * 2u + chunk * 16;
    }
    // The k-step's 128-byte advance goes into the scalar base (kept opaque so that it stays a scalar
    // register pair) and the per-lane part stays a 32-bit offset: the load then needs no vector
    // address arithmetic at all.
    auto step_base = [&](const char* base, int kt) {
        const char* p = base + static_cast<size_t>(kt) * 128;
        asm volatile("" : "+s"(p));
        return p;
    };
    // load i of a stage: i < QA belongs to the A operand (ring slot sa), the others to W (ring slot sw)
    auto dma = [&](int i, int sa, int sw, const char* a_k, const char* w_k) {
#if DICEMOE_FFN_DIAG
        if (DIAG & 2) return;
#endif
        uint32_t off = goff[i];
        asm volatile("" : "+v"(off));          // keeps the zero extension next to the load (scalar base + 32-bit offset form)
        if (i < QA)
            __builtin_amdgcn_global_load_lds(DICEMOE_GLOBAL_PTR(a_k + off),
                                             DICEMOE_LDS_PTR(a_lds + sa * ABYTES + (wave * QA + i) * 1024), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds(DICEMOE_GLOBAL_PTR(w_k + off),
                                             DICEMOE_LDS_PTR(w_lds + sw * WBYTES + (wave * QB + (i - QA)) * 1024), 16, 0, 0);
    };

    // ---- fragment offsets inside an operand's stage: 32-row blocks are 4 KiB apart, k slices differ in the chunk
    int a_off[4], b_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int chunk = kk * 2 + (lane >> 5);
        const int ra = wm * WM + (lane & 31), rb = wn * WN + (lane & 31);
        a_off[kk] = (ra * CH + (chunk ^ chunk_swizzle<CH>(ra))) * 16;
        b_off[kk] = (rb * CH + (chunk ^ chunk_swizzle<CH>(rb))) * 16;
    }

    f32x16_v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    bf16x8_v fr[2][NFRAG];                           // [set][A fragments 0..TM-1, then W fragments]
    auto read_frag = [&](int set, int f, const char* sta, const char* stw, int kk) {
#if DICEMOE_FFN_DIAG
        if (DIAG & 4) return;
#endif
        const char* p = f < TM ? sta + a_off[kk] + f * 4096 : stw + b_off[kk] + (f - TM) * 4096;
        const u32x4_v v = *reinterpret_cast<const u32x4_v*>(p);
        fr[set][f] = *reinterpret_cast<const bf16x8_v*>(&v);
    };
    auto mfma = [&](int set, int m) {
        const int i = m / TN, j = m % TN;           // operands swapped: see store_slab
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[set][TM + j], fr[set][i], acc[i][j], 0, 0, 0);
    };

    // Split reduction: workgroup row blockIdx.y of the grid takes the y-th share of the 64-deep steps and
    // leaves its float sums in partial[y] (a later pass adds the shares in a fixed order).  The launcher
    // guarantees that every share has the steps the ring needs (>= 4 for a three-deep ring).
    const int nk_all = K / 64;
    const int k_begin = static_cast<int>(blockIdx.y) * nk_all / static_cast<int>(gridDim.y);
    const int nk = (static_cast<int>(blockIdx.y) + 1) * nk_all / static_cast<int>(gridDim.y) - k_begin;
    a_base += static_cast<size_t>(k_begin) * 128;
    w_base += static_cast<size_t>(k_begin) * 128;
    // ---- prologue: every stage in flight, first fragments in registers.  The W parts go first: they
    // do not depend on the row index, whose load is still in flight when a gathering kernel gets here.
#pragma unroll
    for (int s = 0; s < WST; ++s) {
        if (s < nk) {
            const char* w_k = step_base(w_base, s);
#pragma unroll
            for (int i = QA; i < QW; ++i) dma(i, 0, s, nullptr, w_k);
        }
    }
#pragma unroll
    for (int s = 0; s < AST; ++s) {
        if (s < nk) {
            const char* a_k = step_base(a_base, s);
#pragma unroll
            for (int i = 0; i < QA; ++i) dma(i, s, 0, a_k, nullptr);
        }
    }
    // loads return in order: stage 0 is complete once its A part is, i.e. when at most the A parts of
    // the younger stages are outstanding
    if (nk >= WST) wait_vmcnt<(AST - 1) * QA>();
    else wait_vmcnt<0>();
    block_barrier();
#pragma unroll
    for (int f = 0; f < NFRAG; ++f) read_frag(0, f, a_lds, w_lds, 0);
#if DICEMOE_FFN_DIAG
    if (DIAG & 4) {
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {
            const u32x4_v v = *reinterpret_cast<const u32x4_v*>(smem + (f < TM ? a_off[0] : b_off[0]) + (f % 4) * 4096);
            fr[0][f] = fr[1][f] = *reinterpret_cast<const bf16x8_v*>(&v);
        }
    }
#endif

    // One 64-deep step kt; its A stage sits in ring slot sa, its W stage in ring slot sw (the rings may
    // differ in depth: the W operand streams from HBM once and gains most from a third stage, the
    // activations come from cache).  After the barrier of this step the slots are drained and take the
    // stages kt+AST (A) and kt+WST (W): the "refill", A loads first, issued in SPREAD parts, one slice
    // each (part 0 beside the last slice, the others beside the first slices of step kt+1), so that the
    // four wavefronts do not push more loads at the texture path than it takes per slice (a full queue
    // stalls MFMA issue).
    //   NEXT:        step kt+1 exists (barrier, first fragments of the next stage)
    //   PEND:        number of this wavefront's loads that may still be in flight at the barrier: those
    //                issued after the loads of stage kt+1 (loads return in order)
    //   REFA, REFW:  the refill of this step has an A part / a W part
    //   CARA, CARW:  the previous step's refill had an A part / a W part (its later parts are issued here)
    constexpr int PART = (QW + SPREAD - 1) / SPREAD;
    constexpr int PER = (PART + NMFMA - 1) / NMFMA;     // loads per MFMA slot; issued in index order, A before W,
                                                        // which is what the PEND counts rely on
    auto step = [&](auto live_tag, int kt, int sa, int sw, auto next_tag, auto pend_tag, auto refa_tag, auto refw_tag,
                    auto cara_tag, auto carw_tag) {
        constexpr bool LIVE = decltype(live_tag)::value;
        constexpr bool NEXT = decltype(next_tag)::value;
        constexpr int PEND = decltype(pend_tag)::value;
        constexpr bool REFA = decltype(refa_tag)::value, REFW = decltype(refw_tag)::value;
        constexpr bool CARA = decltype(cara_tag)::value, CARW = decltype(carw_tag)::value;
        const int sa_nxt = (sa + 1 == AST) ? 0 : sa + 1, sw_nxt = (sw + 1 == WST) ? 0 : sw + 1;
        const int sa_prev = (sa == 0) ? AST - 1 : sa - 1, sw_prev = (sw == 0) ? WST - 1 : sw - 1;
        const char* cur_a = a_lds + sa * ABYTES;
        const char* cur_w = w_lds + sw * WBYTES;
        const char* nxt_a = a_lds + sa_nxt * ABYTES;
        const char* nxt_w = w_lds + sw_nxt * WBYTES;
        const char* a_carry = step_base(a_base, kt - 1 + AST);      // the refill in flight fills the previous step's slots
        const char* w_carry = step_base(w_base, kt - 1 + WST);
        const char* a_refill = step_base(a_base, kt + AST);
        const char* w_refill = step_base(w_base, kt + WST);
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            const int set = kk & 1;
            DICEMOE_SCHED_FENCE();
#pragma unroll
            for (int m = 0; m < NMFMA; ++m) {
                if (LIVE) mfma(set, m);
                DICEMOE_SCHED_FENCE();
                if (LIVE && m < NFRAG) { read_frag(set ^ 1, m, cur_a, cur_w, kk + 1); DICEMOE_SCHED_FENCE(); }
                if ((CARA || CARW) && kk + 1 < SPREAD) {
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const int i = (kk + 1) * PART + m * PER + j;
                        if (m * PER + j < PART && i < QW && (i < QA ? CARA : CARW)) {
                            dma(i, sa_prev, sw_prev, a_carry, w_carry);
                            DICEMOE_SCHED_FENCE();
                        }
                    }
                }
            }
        }
        // last slice: fragments of slice 3 are in set 1
        DICEMOE_SCHED_FENCE();
        if (NEXT) {
            wait_lgkmcnt<0>();                      // every fragment of this stage has been read
            wait_vmcnt<PEND>();                     // my loads of the next stage have landed
            block_barrier();
        }
        DICEMOE_SCHED_FENCE();
#pragma unroll
        for (int m = 0; m < NMFMA; ++m) {
            if (LIVE) mfma(1, m);
            DICEMOE_SCHED_FENCE();
            if (LIVE && NEXT && m < NFRAG) { read_frag(0, m, nxt_a, nxt_w, 0); DICEMOE_SCHED_FENCE(); }
            if (REFA || REFW) {
#pragma unroll
                for (int j = 0; j < PER; ++j) {
                    const int i = m * PER + j;
                    if (i < PART && i < QW && (i < QA ? REFA : REFW)) { dma(i, sa, sw, a_refill, w_refill); DICEMOE_SCHED_FENCE(); }
                }
            }
        }
    };
    const std::true_type yes{};
    const std::false_type no{};
    const std::integral_constant<int, 0> p0{};
    // A wavefront whose 32 TM rows all lie past the end of the segment (the ragged last row tile of an
    // expert) has nothing to compute: it keeps its share of the loads, the waits and the barriers, and
    // leaves the matrix pipe of its SIMD to the wavefront it shares it with.
    const bool live = row0 + wm * WM < row_end;
    auto run_steps = [&](auto live_tag) {
        int sa = 0, sw = 0;
        auto advance = [&]() { sa = (sa + 1 == AST) ? 0 : sa + 1; sw = (sw + 1 == WST) ? 0 : sw + 1; };
        // Which loads are younger than those of stage kt+1 at the barrier of step kt follows from the issue
        // order: prologue W0.. then A0..; refill of step j: A(j+AST) then W(j+WST).
        if (AST == 2 && WST == 2) {
            if (nk == 1) {
                step(live_tag, 0, 0, 0, no, p0, no, no, no, no);
            } else {
                if (nk > 2) step(live_tag, 0, 0, 0, yes, p0, yes, yes, no, no); else step(live_tag, 0, 0, 0, yes, p0, no, no, no, no);
                advance();
                int kt = 1;
                for (; kt + 2 < nk; ++kt) { step(live_tag, kt, sa, sw, yes, p0, yes, yes, yes, yes); advance(); }
                if (nk > 2) { step(live_tag, kt, sa, sw, yes, p0, no, no, yes, yes); advance(); ++kt; }
                step(live_tag, kt, sa, sw, no, p0, no, no, no, no);
            }
        } else if (AST == 2 && WST == 3) {
            const std::integral_constant<int, QB> pw{};      // the W part of the previous step's refill
            step(live_tag, 0, 0, 0, yes, p0, yes, yes, no, no);
            advance();
            int kt = 1;
            for (; kt + 3 < nk; ++kt) { step(live_tag, kt, sa, sw, yes, pw, yes, yes, yes, yes); advance(); }
            step(live_tag, kt, sa, sw, yes, pw, yes, no, yes, yes); advance(); ++kt;      // kt = nk-3: A(nk-1) is the last refill
            step(live_tag, kt, sa, sw, yes, p0, no, no, yes, no); advance(); ++kt;        // kt = nk-2
            step(live_tag, kt, sa, sw, no, p0, no, no, no, no);                           // kt = nk-1
        } else if (AST == 2 && WST == 4) {
            // as (2,3) with one more weight stage in flight: at the barrier of step kt the youngest load still
            // needed is the A part of the previous refill, and only that refill's W part is younger
            const std::integral_constant<int, QB> pw{};
            step(live_tag, 0, 0, 0, yes, p0, yes, yes, no, no);
            advance();
            int kt = 1;
            for (; kt + 4 < nk; ++kt) { step(live_tag, kt, sa, sw, yes, pw, yes, yes, yes, yes); advance(); }
            step(live_tag, kt, sa, sw, yes, pw, yes, no, yes, yes); advance(); ++kt;      // kt = nk-4: W(nk-1) went with the refill before
            step(live_tag, kt, sa, sw, yes, p0, yes, no, yes, no); advance(); ++kt;       // kt = nk-3: A(nk-1) is the last refill
            step(live_tag, kt, sa, sw, yes, p0, no, no, yes, no); advance(); ++kt;        // kt = nk-2
            step(live_tag, kt, sa, sw, no, p0, no, no, no, no);                           // kt = nk-1
        } else if (AST == 4 && WST == 4) {
            // three stages in flight per operand.  Loads younger than stage kt+1 at the barrier of step kt:
            // step 0: A2, A3 of the prologue; step 1: A3 and refill 0; later: the last two refills
            const std::integral_constant<int, 2 * QA> p2a{};
            const std::integral_constant<int, QA + QW> paq{};
            const std::integral_constant<int, 2 * QW> p2q{};
            const std::integral_constant<int, QW> pq{};
            step(live_tag, 0, 0, 0, yes, p2a, yes, yes, no, no);
            advance();
            step(live_tag, 1, sa, sw, yes, paq, yes, yes, yes, yes);
            advance();
            int kt = 2;
            for (; kt + 4 < nk; ++kt) { step(live_tag, kt, sa, sw, yes, p2q, yes, yes, yes, yes); advance(); }
            step(live_tag, kt, sa, sw, yes, p2q, no, no, yes, yes); advance(); ++kt;      // kt = nk-4: the last refill was issued at nk-5
            step(live_tag, kt, sa, sw, yes, pq, no, no, no, no); advance(); ++kt;         // kt = nk-3
            step(live_tag, kt, sa, sw, yes, p0, no, no, no, no); advance(); ++kt;         // kt = nk-2
            step(live_tag, kt, sa, sw, no, p0, no, no, no, no);                           // kt = nk-1
        } else {
            const std::integral_constant<int, QA> pa{};      // step 0: the prologue issued the A parts last
            const std::integral_constant<int, QW> pq{};      // the previous step's whole refill
            step(live_tag, 0, 0, 0, yes, pa, yes, yes, no, no);
            advance();
            int kt = 1;
            for (; kt + 3 < nk; ++kt) { step(live_tag, kt, sa, sw, yes, pq, yes, yes, yes, yes); advance(); }
            step(live_tag, kt, sa, sw, yes, pq, no, no, yes, yes); advance(); ++kt;       // kt = nk-3
            step(live_tag, kt, sa, sw, yes, p0, no, no, no, no); advance(); ++kt;         // kt = nk-2
            step(live_tag, kt, sa, sw, no, p0, no, no, no, no);                           // kt = nk-1
        }

    };
    if (live) run_steps(yes);
    else run_steps(no);

    // ---- epilogue: the stage buffers are free once every wavefront is past its last fragment read
    wait_vmcnt<0>();
    wait_lgkmcnt<0>();
    block_barrier();
    if (!live) return;
#if DICEMOE_FFN_DIAG
    if (DIAG & 1) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) s += acc[i][j][v];
        if (s == 1234.5f) C[0] = 1;
        return;
    }
#endif
    if (partial) {
        // raw sums of this share: lane (m, h) holds, per 32 x 32 block, columns 8g + 4h .. + 3 of row m
        float* dst = partial + static_cast<size_t>(blockIdx.y) * partial_rows * N;
        const int m_local = lane & 31, h = lane >> 5;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = row0 + wm * WM + i * 32 + m_local;
            if (r >= row_end || r >= partial_rows) continue;      // (the second: a caller whose max_rows is too small)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = col_first + j * 32 + 8 * g + 4 * h;
                    if (n < N)
                        *reinterpret_cast<f32x4_v*>(dst + static_cast<size_t>(r) * N + n) =
                            f32x4_v{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                }
        }
        return;
    }
    char* region = smem + wave * REGION;
    float* bias_lds = reinterpret_cast<float*>(region + slab_bytes<TN>());
    stage_bias<WN>(bias_reg, bias_lds, lane);
    float4 bias_groups[TN][4];
    read_bias_groups<TN>(bias_lds, lane, bias_groups);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (GELU)      // the GELU epilogue is bound by its arithmetic: storing straight from registers saves the LDS trip
            store_slab_direct<TN, GELU>(acc[i], bias_groups, C, N, row0 + wm * WM + i * 32, row_end, col_first, lane, out_index);
        else
            store_slab<TN, GELU>(acc[i], region, bias_groups, C, N, row0 + wm * WM + i * 32, row_end, col_first, lane,
                                 out_index);
    }
}

// The wide kernels use more dynamic LDS than a launch may ask for by default; the limit is a
// per-device attribute of each kernel, raised by prepare_expert_ffn() before the first launch on a device.
template <int TM, int TN, int SPREAD, int AST, int WST, bool GELU, int WGM = 2, int WGN = 2>
static hipError_t configure_gemm_bf16_wide()
{
    constexpr int smem = (AST * 32 * TM * WGM + WST * 32 * TN * WGN) * 128;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_gemm_bf16_wide_kernel<TM, TN, SPREAD, AST, WST, GELU, WGM, WGN>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, smem);
}

template <int TM, int TN, int SPREAD, int AST, int WST, bool GELU, int WGM = 2, int WGN = 2>
static hipError_t launch_gemm_bf16_wide(const void* A, const void* W, const float* bias, void* C, int N, int K,
                                        const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg,
                                        int max_rows, hipStream_t stream, const int32_t* row_index = nullptr,
                                        int row_div = 1, const int32_t* out_index = nullptr, int by_expert = 0,
                                        float* partial = nullptr, int k_splits = 1, int32_t* status = nullptr)
{
    constexpr int BM = 32 * TM * WGM, BN = 32 * TN * WGN;
    auto kern = ffn_gemm_bf16_wide_kernel<TM, TN, SPREAD, AST, WST, GELU, WGM, WGN>;
    constexpr int smem = (AST * BM + WST * BN) * 128;
    if (k_splits < 1 || (k_splits > 1 && (!partial || GELU))) return hipErrorInvalidValue;
    const int nk_min = K / 64 / k_splits;                         // steps of the smallest share
    if (WST == 3 && nk_min < 4) return hipErrorInvalidValue;      // the three-deep loops are written for at least four steps
    if (WST == 4 && nk_min < (AST == 4 ? 7 : 5)) return hipErrorInvalidValue;      // the four-deep loops: at least seven (five) steps
    if (nk_min < 1) return hipErrorInvalidValue;
    const int n_tiles_n = (N + BN - 1) / BN;
    const int m_tiles = (max_rows + BM - 1) / BM + n_seg;
    const int bands = (m_tiles + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(bands) * 8 * n_tiles_n, static_cast<unsigned>(k_splits)),
                       dim3(64 * WGM * WGN), smem, stream,
                       static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(W), bias, static_cast<bf16_t*>(C), N,
                       K, seg_offsets, seg_expert, n_seg, n_tiles_n, m_tiles, row_index, row_div, out_index, by_expert,
                       k_splits > 1 ? partial : nullptr, max_rows, status);
    return hipGetLastError();
}

}  // namespace dicemoe
