// Dispatch on one device (Algorithm 1, "x_d <- all2all_dispatch(x, idx)"): group the refreshed
// (token, slot) pairs by destination expert with a stable counting sort, then gather the token
// rows into the expert-contiguous buffer.
//
// dispatch_index_kernel: one workgroup of 16 wavefronts.  Wave w owns the contiguous range of
// pair ids [w*L, (w+1)*L), so "wave-major, then lane order" is ascending pair id and the sort is
// stable by construction.  Lanes that hold the same expert find each other with six ballots (one
// per bit of the expert id); the lowest such lane keeps a per-wave, per-expert running count in
// LDS.  Phase A counts (and remembers each pair's rank inside its wave-and-expert group), a scan
// over (expert, wave) turns the counts into bases, phase B adds base and rank and writes perm / inv
// (for ranges too long for registers it walks the range again instead).  All integer work, no
// atomics: the result is unique.
//
// dispatch_gather_kernel: one wavefront per token reads the row once (16 bytes per lane per
// pass) and stores it to each of its refreshed slots' packed rows; bound by HBM traffic
// T*d*b read + R*d*b written.
#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

constexpr int kIdxThreads = 1024;
constexpr int kIdxWaves = kIdxThreads / kWave;

// order this wavefront's LDS accesses: reads before the point complete before writes after it
// are issued, and the compiler keeps them on their side
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// lanes of this wave that are live and hold the same expert id as the calling lane; nbits = number of
// bits an expert id can have (ballots are scalar work, and one scalar unit serves the whole workgroup)
__device__ __forceinline__ uint64_t same_expert_peers(bool live, int e, int nbits) {
    uint64_t peers = __ballot(live);
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        if (b < nbits) {                          // uniform
            const bool bit = (e >> b) & 1;
            const uint64_t bb = __ballot(bit);
            peers &= bit ? bb : ~bb;
        }
    }
    return peers;
}

constexpr int kChunk = 8;

// Expert ids of one chunk of this wave's pairs, -1 where the pair is past the range, not refreshed
// or carries a bad id.  The loads are unconditional (index clamped into the range) so that the
// whole chunk is in flight at once.
__device__ __forceinline__ void load_chunk(const int32_t* __restrict__ expert_idx, const uint8_t* __restrict__ mask,
                                           int c0, int lane, int hi, int E, int (&ev)[kChunk]) {
    uint8_t mv[kChunk];
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
        const int p = c0 + u * kWave + lane;
        ev[u] = expert_idx[p < hi ? p : hi - 1];
    }
    if (mask != nullptr) {
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int p = c0 + u * kWave + lane;
            mv[u] = mask[p < hi ? p : hi - 1];
        }
    } else {
#pragma unroll
        for (int u = 0; u < kChunk; ++u) mv[u] = 1;
    }
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
        const int p = c0 + u * kWave + lane;
        const bool ok = p < hi && mv[u] != 0 && static_cast<unsigned>(ev[u]) < static_cast<unsigned>(E);
        ev[u] = ok ? ev[u] : -1;
    }
}

// MAXC > 0: the wave's whole range fits in MAXC chunks, so the expert ids and the rank of every pair
// inside its (wave, expert) group stay in registers between the counting pass and the placement:
// one pass of loads and ballots instead of two.  MAXC == 0: any N, two passes over global memory.
template <int MAXC>
__global__ __launch_bounds__(kIdxThreads) void dispatch_index_kernel(const int32_t* __restrict__ expert_idx,
                                                                    const uint8_t* __restrict__ mask, int N, int E,
                                                                    int32_t* __restrict__ counts,
                                                                    int32_t* __restrict__ offsets,
                                                                    int32_t* __restrict__ perm,
                                                                    int32_t* __restrict__ inv)
{
    __shared__ int wave_run[kIdxWaves][kMaxExperts];  // counts, then running bases
    __shared__ int s_cnt[kMaxExperts];
    __shared__ int s_off[kMaxExperts + 1];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = lane_id();
    const int nbits = E > 1 ? 32 - __builtin_clz(static_cast<unsigned>(E - 1)) : 0;
    const int L = (((N + kIdxWaves - 1) / kIdxWaves) + kWave - 1) / kWave * kWave;
    const int lo = wave * L;
    const int hi = (lo + L < N) ? lo + L : N;

    wave_run[tid / kMaxExperts][tid % kMaxExperts] = 0;   // 1024 threads cover the 16 x 64 table
    __syncthreads();

    constexpr int NC = MAXC > 0 ? MAXC : 1;
    int ev_keep[NC][kChunk];      // expert id, -1 if not live
    int rank_keep[NC][kChunk];    // pairs of the same wave and expert before this one

    // Both phases walk the range in chunks of kChunk wave-wide steps: all loads of a chunk are
    // issued first (they are independent), then the steps are processed from registers in order.
    // phase A: per-wave, per-expert counts of refreshed pairs
    if (MAXC > 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int c0 = lo + c * kWave * kChunk;
            if (c0 < hi) {                                 // wave-uniform
                load_chunk(expert_idx, mask, c0, lane, hi, E, ev_keep[c]);
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    const bool live = ev_keep[c][u] >= 0;
                    const int e = live ? ev_keep[c][u] : 0;
                    const uint64_t peers = same_expert_peers(live, e, nbits);
                    const int before = __popcll(peers & lanemask_lt());
                    const int run = wave_run[wave][e];     // every peer reads the same running count ...
                    rank_keep[c][u] = run + before;
                    wave_sync();
                    if (live && before == 0) wave_run[wave][e] = run + __popcll(peers);   // ... then the first updates it
                    wave_sync();
                }
            } else {
#pragma unroll
                for (int u = 0; u < kChunk; ++u) { ev_keep[c][u] = -1; rank_keep[c][u] = 0; }
            }
        }
    } else {
        for (int c0 = lo; c0 < hi; c0 += kWave * kChunk) {
            int ev[kChunk];
            load_chunk(expert_idx, mask, c0, lane, hi, E, ev);
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const bool live = ev[u] >= 0;
                const int e = live ? ev[u] : 0;
                const uint64_t peers = same_expert_peers(live, e, nbits);
                if (live && (peers & lanemask_lt()) == 0) wave_run[wave][e] = wave_run[wave][e] + __popcll(peers);
                wave_sync();
            }
        }
    }
    __syncthreads();

    // exclusive scan over waves for each expert; then over experts
    if (tid < E) {
        int run = 0;
        for (int w = 0; w < kIdxWaves; ++w) {
            const int c = wave_run[w][tid];
            wave_run[w][tid] = run;
            run += c;
        }
        s_cnt[tid] = run;
        counts[tid] = run;
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) { s_off[e] = run; offsets[e] = run; run += s_cnt[e]; }
        s_off[E] = run;
        offsets[E] = run;
    }
    __syncthreads();
    const int R = s_off[E];

    // phase B: final positions
    if (MAXC > 0) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int c0 = lo + c * kWave * kChunk;
            if (c0 < hi) {
#pragma unroll
                for (int u = 0; u < kChunk; ++u) {
                    const int p = c0 + u * kWave + lane;
                    const int e = ev_keep[c][u];
                    int r = -1;
                    if (e >= 0) {
                        r = s_off[e] + wave_run[wave][e] + rank_keep[c][u];
                        perm[r] = p;
                    }
                    if (p < hi) inv[p] = r;
                }
            }
        }
    } else {
        for (int c0 = lo; c0 < hi; c0 += kWave * kChunk) {
            int ev[kChunk];
            load_chunk(expert_idx, mask, c0, lane, hi, E, ev);
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const int p = c0 + u * kWave + lane;
                const bool live = ev[u] >= 0;
                const int e = live ? ev[u] : 0;
                const uint64_t peers = same_expert_peers(live, e, nbits);
                const int before = __popcll(peers & lanemask_lt());
                int r = -1;
                if (live) r = s_off[e] + wave_run[wave][e] + before;
                wave_sync();
                if (live && before == 0) wave_run[wave][e] = wave_run[wave][e] + __popcll(peers);
                wave_sync();
                if (live) perm[r] = p;
                if (p < hi) inv[p] = r;
            }
        }
    }
    for (int r = R + tid; r < N; r += kIdxThreads) perm[r] = -1;
}

template <typename T>
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const T* __restrict__ x, const int32_t* __restrict__ inv,
                                                              int T_tok, int d, int k, T* __restrict__ x_packed)
{
    constexpr int V = Store<T>::kVec;
    const int tok = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tok >= T_tok) return;
    const int lane = lane_id();
    const int nvec = d / V;
    const int32_t* rows = inv + static_cast<size_t>(tok) * k;
    bool any = false;
    for (int j = 0; j < k; ++j) any |= rows[j] >= 0;
    if (!any) return;
    const uint4* src = reinterpret_cast<const uint4*>(x + static_cast<size_t>(tok) * d);
    uint4* dst = reinterpret_cast<uint4*>(x_packed);
    for (int c = lane; c < nvec; c += kWave) {
        const uint4 v = src[c];
        for (int j = 0; j < k; ++j) {
            const int r = rows[j];
            if (r >= 0) dst[static_cast<size_t>(r) * nvec + c] = v;
        }
    }
}

hipError_t launch_dispatch(bool bf16, const void* x, const int32_t* idx, const uint8_t* mask, int T_tok, int d,
                           int E, int k, void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm,
                           int32_t* inv, hipStream_t stream)
{
    const int N = T_tok * k;
    // pairs per wave, rounded up to whole wave-wide steps; up to 4 chunks of them stay in registers
    const int per_wave = (((N + kIdxWaves - 1) / kIdxWaves) + kWave - 1) / kWave * kWave;
    if (per_wave <= kWave * kChunk)
        hipLaunchKernelGGL(dispatch_index_kernel<1>, dim3(1), dim3(kIdxThreads), 0, stream, idx, mask, N, E, counts,
                           offsets, perm, inv);
    else if (per_wave <= 2 * kWave * kChunk)
        hipLaunchKernelGGL(dispatch_index_kernel<2>, dim3(1), dim3(kIdxThreads), 0, stream, idx, mask, N, E, counts,
                           offsets, perm, inv);
    else if (per_wave <= 4 * kWave * kChunk)
        hipLaunchKernelGGL(dispatch_index_kernel<4>, dim3(1), dim3(kIdxThreads), 0, stream, idx, mask, N, E, counts,
                           offsets, perm, inv);
    else
        hipLaunchKernelGGL(dispatch_index_kernel<0>, dim3(1), dim3(kIdxThreads), 0, stream, idx, mask, N, E, counts,
                           offsets, perm, inv);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || T_tok == 0 || x_packed == nullptr) return err;   // no packed buffer: index only
    const int blocks = (T_tok + 3) / 4;
    if (bf16)
        hipLaunchKernelGGL(dispatch_gather_kernel<bf16_t>, dim3(blocks), dim3(256), 0, stream,
                           static_cast<const bf16_t*>(x), inv, T_tok, d, k, static_cast<bf16_t*>(x_packed));
    else
        hipLaunchKernelGGL(dispatch_gather_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                           static_cast<const float*>(x), inv, T_tok, d, k, static_cast<float*>(x_packed));
    return hipGetLastError();
}

__global__ void ep_segments_kernel(const int32_t* __restrict__ recv_counts, int n_seg, int E_loc,
                                   int32_t* __restrict__ seg_offsets, int32_t* __restrict__ seg_expert)
{
    // tiny table (at most 1024 entries): one thread walks it
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        int run = 0;
        for (int g = 0; g < n_seg; ++g) {
            seg_offsets[g] = run;
            seg_expert[g] = g % E_loc;
            run += recv_counts[g];
        }
        seg_offsets[n_seg] = run;
    }
}

hipError_t launch_ep_segments(const int32_t* recv_counts, int n_seg, int E_loc, int32_t* seg_offsets,
                              int32_t* seg_expert, hipStream_t stream)
{
    hipLaunchKernelGGL(ep_segments_kernel, dim3(1), dim3(64), 0, stream, recv_counts, n_seg, E_loc, seg_offsets,
                       seg_expert);
    return hipGetLastError();
}

}  // namespace dicemoe
