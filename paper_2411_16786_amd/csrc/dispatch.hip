// Dispatch on one device (Algorithm 1, "x_d <- all2all_dispatch(x, idx)"): group the refreshed
// (token, slot) pairs by destination expert with a stable counting sort, then gather the token
// rows into the expert-contiguous buffer.
//
// Index kernels (count, then place; no workgroup waits for another).  Workgroup b owns the
// contiguous pair ids [b*256*S, (b+1)*256*S), wave w of it a contiguous quarter, and a wave walks
// its range in steps of 64, so "workgroup, wave, step, lane" is ascending pair id and the sort is
// stable by construction.
//   dispatch_count_kernel: per-workgroup, per-expert counts of refreshed pairs -> scratch[b][e].
//   dispatch_place_kernel: every workgroup sums the scratch table into the experts' totals and
//     into the counts of the workgroups before it (grids beyond 256 workgroups: dispatch_scan_kernel
//     has done that once for all of them), scans the totals into the experts' offsets,
//     ranks its own pairs (lanes that hold the same expert find each other with one ballot per bit
//     of the expert id; per-wave, per-expert running counts in LDS), and writes perm / inv.
//     With a single workgroup the table is not needed and the count kernel is not launched.
// All integer work; the only atomics are integer adds in LDS: the result is unique.
//
// dispatch_gather_kernel: one wavefront per token reads the row once (16 bytes per lane per
// pass) and stores it to each of its refreshed slots' packed rows; bound by HBM traffic
// T*d*b read + R*d*b written.
#include <mutex>

#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

constexpr int kIdxThreads = 256;
constexpr int kIdxWaves = kIdxThreads / kWave;

// order this wavefront's LDS accesses: reads before the point complete before writes after it
// are issued, and the compiler keeps them on their side
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// lanes of this wave that are live and hold the same expert id as the calling lane; nbits = number of
// bits an expert id can have (ballots are scalar work)
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

// Expert ids of this wave's S steps, -1 where the pair is past the end, not refreshed or carries a
// bad id.  The loads are unconditional (index clamped) so that all of them are in flight at once.
template <int S>
__device__ __forceinline__ void load_steps(const int32_t* __restrict__ expert_idx, const uint8_t* __restrict__ mask,
                                           int p0, int lane, int N, int E, int (&ev)[S]) {
    uint8_t mv[S];
#pragma unroll
    for (int u = 0; u < S; ++u) {
        const int p = p0 + u * kWave + lane;
        ev[u] = expert_idx[p < N ? p : N - 1];
    }
    if (mask != nullptr) {
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const int p = p0 + u * kWave + lane;
            mv[u] = mask[p < N ? p : N - 1];
        }
    } else {
#pragma unroll
        for (int u = 0; u < S; ++u) mv[u] = 1;
    }
#pragma unroll
    for (int u = 0; u < S; ++u) {
        const int p = p0 + u * kWave + lane;
        const bool ok = p < N && mv[u] != 0 && static_cast<unsigned>(ev[u]) < static_cast<unsigned>(E);
        ev[u] = ok ? ev[u] : -1;
    }
}

template <int S>
__global__ __launch_bounds__(kIdxThreads) void dispatch_count_kernel(const int32_t* __restrict__ expert_idx,
                                                                    const uint8_t* __restrict__ mask, int N, int E,
                                                                    int32_t* __restrict__ block_counts)
{
    __shared__ int cnt[kMaxExperts];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = lane_id();
    const int nbits = E > 1 ? 32 - __builtin_clz(static_cast<unsigned>(E - 1)) : 0;
    if (tid < kMaxExperts) cnt[tid] = 0;
    __syncthreads();
    const int p0 = (static_cast<int>(blockIdx.x) * kIdxWaves + wave) * kWave * S;
    if (p0 < N) {                                           // wave-uniform
        int ev[S];
        load_steps<S>(expert_idx, mask, p0, lane, N, E, ev);
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const bool live = ev[u] >= 0;
            const int e = live ? ev[u] : 0;
            const uint64_t peers = same_expert_peers(live, e, nbits);
            if (live && (peers & lanemask_lt()) == 0) atomicAdd(&cnt[e], __popcll(peers));   // one add per expert and step
        }
    }
    __syncthreads();
    if (tid < E) block_counts[static_cast<size_t>(blockIdx.x) * E + tid] = cnt[tid];
}

// Grids beyond 256 workgroups: one workgroup turns the table of per-workgroup counts into exclusive
// prefixes over the workgroups (row b: pairs of each expert in the workgroups before b) and appends the
// totals as row n_blocks, so that every placing workgroup reads two rows instead of the whole table.
// Wave w takes experts w, w + 16, ...; lane l of it owns a contiguous run of workgroups.
__global__ __launch_bounds__(1024) void dispatch_scan_kernel(int32_t* __restrict__ block_counts, int n_blocks, int E)
{
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    const int per_lane = (n_blocks + kWave - 1) / kWave;
    const int b_lo = lane * per_lane;
    const int b_hi = (b_lo + per_lane < n_blocks) ? b_lo + per_lane : n_blocks;
    for (int e = wave; e < E; e += 1024 / kWave) {
        int run = 0;
        for (int bb = b_lo; bb < b_hi; ++bb) run += block_counts[static_cast<size_t>(bb) * E + e];
        int incl = run;                           // inclusive scan of the lanes' sums
#pragma unroll
        for (int sh = 1; sh < kWave; sh <<= 1) {
            const int v = __shfl_up(incl, sh, kWave);
            if (lane >= sh) incl += v;
        }
        int prefix = incl - run;
        for (int bb = b_lo; bb < b_hi; ++bb) {
            const int c = block_counts[static_cast<size_t>(bb) * E + e];
            block_counts[static_cast<size_t>(bb) * E + e] = prefix;
            prefix += c;
        }
        if (lane == kWave - 1) block_counts[static_cast<size_t>(n_blocks) * E + e] = incl;
    }
}

template <int S>
__global__ __launch_bounds__(kIdxThreads) void dispatch_place_kernel(const int32_t* __restrict__ expert_idx,
                                                                    const uint8_t* __restrict__ mask, int N, int E,
                                                                    const int32_t* __restrict__ block_counts,
                                                                    int prefix_ready, int32_t* __restrict__ counts,
                                                                    int32_t* __restrict__ offsets,
                                                                    int32_t* __restrict__ perm,
                                                                    int32_t* __restrict__ inv)
{
    __shared__ int wave_run[kIdxWaves][kMaxExperts];   // running count of a wave's pairs per expert; at the end its total
    __shared__ int s_tot[kMaxExperts];                 // pairs per expert over all workgroups
    __shared__ int s_pre[kMaxExperts];                 // pairs per expert in the workgroups before this one
    __shared__ int s_off[kMaxExperts + 1];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = lane_id();
    const int b = blockIdx.x;
    const int n_blocks = gridDim.x;
    const int nbits = E > 1 ? 32 - __builtin_clz(static_cast<unsigned>(E - 1)) : 0;
    wave_run[tid / kMaxExperts][tid % kMaxExperts] = 0;   // 256 threads cover the 4 x 64 table
    if (tid < kMaxExperts) { s_tot[tid] = 0; s_pre[tid] = 0; }
    __syncthreads();

    // the table of the other workgroups' counts: totals, and the part that precedes this workgroup.  Large
    // grids (prefix_ready) find both already summed by dispatch_scan_kernel: row b holds the counts of the
    // workgroups before b, row n_blocks the totals.
    if (n_blocks > 1 && prefix_ready) {
        if (tid < E) {
            s_pre[tid] = block_counts[static_cast<size_t>(b) * E + tid];
            s_tot[tid] = block_counts[static_cast<size_t>(n_blocks) * E + tid];
        }
    } else if (n_blocks > 1) {
        for (int i = tid; i < n_blocks * E; i += kIdxThreads) {
            const int c = block_counts[i];
            const int bb = i / E, e = i - bb * E;
            if (c != 0) {
                atomicAdd(&s_tot[e], c);
                if (bb < b) atomicAdd(&s_pre[e], c);
            }
        }
    }

    // rank of each of this wave's pairs among the wave's pairs of the same expert
    const int p0 = (b * kIdxWaves + wave) * kWave * S;
    int ev[S], rank[S];
    if (p0 < N) {                                           // wave-uniform
        load_steps<S>(expert_idx, mask, p0, lane, N, E, ev);
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const bool live = ev[u] >= 0;
            const int e = live ? ev[u] : 0;
            const uint64_t peers = same_expert_peers(live, e, nbits);
            const int before = __popcll(peers & lanemask_lt());
            const int run = wave_run[wave][e];             // every peer reads the same running count ...
            rank[u] = run + before;
            wave_sync();
            if (live && before == 0) wave_run[wave][e] = run + __popcll(peers);   // ... then the first updates it
            wave_sync();
        }
    } else {
#pragma unroll
        for (int u = 0; u < S; ++u) { ev[u] = -1; rank[u] = 0; }
    }
    __syncthreads();
    if (n_blocks == 1 && tid < E) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kIdxWaves; ++w) t += wave_run[w][tid];
        s_tot[tid] = t;
    }
    __syncthreads();
    // exclusive scan over the experts: lane e of the first wave holds expert e's total
    if (wave == 0) {
        const int mine = lane < E ? s_tot[lane] : 0;
        int incl = mine;
#pragma unroll
        for (int sh = 1; sh < kWave; sh <<= 1) {
            const int v = __shfl_up(incl, sh, kWave);
            if (lane >= sh) incl += v;
        }
        if (lane < E) {
            s_off[lane] = incl - mine;
            if (b == 0) { counts[lane] = mine; offsets[lane] = incl - mine; }
        }
        if (lane == E - 1) {
            s_off[E] = incl;
            if (b == 0) offsets[E] = incl;
        }
    }
    __syncthreads();
    const int R = s_off[E];

    if (p0 < N) {
#pragma unroll
        for (int u = 0; u < S; ++u) {
            const int p = p0 + u * kWave + lane;
            const int e = ev[u];
            int r = -1;
            if (e >= 0) {
                int base = s_off[e] + s_pre[e];
                for (int w = 0; w < wave; ++w) base += wave_run[w][e];
                r = base + rank[u];
                perm[r] = p;
            }
            if (p < N) {
                inv[p] = r;
                if (p >= R) perm[p] = -1;                  // packed rows beyond the refreshed ones
            }
        }
    }
}

// NP > 0: a row is at most NP passes of 64 lanes x 16 bytes; all passes are loaded before the first
// store (one memory round trip per token); NP == 0: any row length, pass by pass.
template <typename T, int NP>
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const T* __restrict__ x, const int32_t* __restrict__ inv,
                                                              int T_tok, int d, int k, int all_pairs, T* __restrict__ x_packed)
{
    constexpr int V = Store<T>::kVec;
    const int tok = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tok >= T_tok) return;
    const int lane = lane_id();
    const int nvec = d / V;
    const int32_t* rows = inv + static_cast<size_t>(tok) * k;
    const u32x4_t* src = reinterpret_cast<const u32x4_t*>(x + static_cast<size_t>(tok) * d);
    u32x4_t* dst = reinterpret_cast<u32x4_t*>(x_packed);
    if (NP > 0 && all_pairs) {
        // every pair is refreshed: the row is needed whatever inv says, so its loads go out together with
        // the loads of the destinations instead of behind them
        constexpr int NPN = NP > 0 ? NP : 1;
        u32x4_t v[NPN];
#pragma unroll
        for (int p = 0; p < NPN; ++p) {
            const int c = lane + p * kWave;
            v[p] = c < nvec ? src[c] : u32x4_t{0u, 0u, 0u, 0u};
        }
        for (int j = 0; j < k; ++j) {
            const int r = rows[j];
            if (r < 0) continue;
#pragma unroll
            for (int p = 0; p < NPN; ++p) {
                const int c = lane + p * kWave;
                if (c < nvec) dst[static_cast<size_t>(r) * nvec + c] = v[p];
            }
        }
        return;
    }
    bool any = false;
    for (int j = 0; j < k; ++j) any |= rows[j] >= 0;
    if (!any) return;
    if (NP > 0) {
        constexpr int NPN = NP > 0 ? NP : 1;
        u32x4_t v[NPN];
#pragma unroll
        for (int p = 0; p < NPN; ++p) {
            const int c = lane + p * kWave;
            v[p] = c < nvec ? src[c] : u32x4_t{0u, 0u, 0u, 0u};
        }
        for (int j = 0; j < k; ++j) {
            const int r = rows[j];
            if (r < 0) continue;
#pragma unroll
            for (int p = 0; p < NPN; ++p) {
                const int c = lane + p * kWave;
                if (c < nvec) dst[static_cast<size_t>(r) * nvec + c] = v[p];
            }
        }
    } else {
        for (int c = lane; c < nvec; c += kWave) {
            const u32x4_t v = src[c];
            for (int j = 0; j < k; ++j) {
                const int r = rows[j];
                if (r >= 0) dst[static_cast<size_t>(r) * nvec + c] = v;
            }
        }
    }
}

// Steps per wave and workgroups of the index kernels for N pairs.  Up to 2048 pairs one workgroup
// sorts alone (one launch); beyond, the fewest steps (1, 2, 4, 8) that keep the grid at 256 workgroups
// or fewer; beyond 2^19 pairs the grid grows instead.
static void dispatch_plan(long long N, int& steps, int& blocks)
{
    steps = 1;
    if (N <= 8 * kIdxThreads) {
        while (static_cast<long long>(kIdxThreads) * steps < N) steps *= 2;
        blocks = 1;
        return;
    }
    while (steps < 8 && (N + static_cast<long long>(kIdxThreads) * steps - 1) / (kIdxThreads * steps) > 256) steps *= 2;
    const long long b = (N + static_cast<long long>(kIdxThreads) * steps - 1) / (kIdxThreads * steps);
    blocks = b > 0 ? static_cast<int>(b) : 1;
}

size_t dispatch_scratch_bytes(long long n_pairs, int E)
{
    int steps, blocks;
    dispatch_plan(n_pairs, steps, blocks);
    return blocks > 1 ? static_cast<size_t>(blocks + 1) * E * sizeof(int32_t) : 0;      // one row per workgroup, and the totals
}

template <int S>
static void launch_dispatch_index(const int32_t* idx, const uint8_t* mask, int N, int E, int blocks, int32_t* scratch,
                                  int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv, hipStream_t stream)
{
    const int scan = blocks > 256 ? 1 : 0;      // small grids: every placing workgroup sums the table itself
    if (blocks > 1)
        hipLaunchKernelGGL(dispatch_count_kernel<S>, dim3(blocks), dim3(kIdxThreads), 0, stream, idx, mask, N, E, scratch);
    if (scan)
        hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(1024), 0, stream, scratch, blocks, E);
    hipLaunchKernelGGL(dispatch_place_kernel<S>, dim3(blocks), dim3(kIdxThreads), 0, stream, idx, mask, N, E, scratch,
                       scan, counts, offsets, perm, inv);
}

hipError_t launch_dispatch(bool bf16, const void* x, const int32_t* idx, const uint8_t* mask, int T_tok, int d,
                           int E, int k, void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm,
                           int32_t* inv, int32_t* scratch, hipStream_t stream)
{
    const int N = T_tok * k;
    int steps, blocks;
    dispatch_plan(N, steps, blocks);
    if (blocks > 1 && scratch == nullptr) return hipErrorInvalidValue;
    switch (steps) {
    case 1: launch_dispatch_index<1>(idx, mask, N, E, blocks, scratch, counts, offsets, perm, inv, stream); break;
    case 2: launch_dispatch_index<2>(idx, mask, N, E, blocks, scratch, counts, offsets, perm, inv, stream); break;
    case 4: launch_dispatch_index<4>(idx, mask, N, E, blocks, scratch, counts, offsets, perm, inv, stream); break;
    default: launch_dispatch_index<8>(idx, mask, N, E, blocks, scratch, counts, offsets, perm, inv, stream); break;
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || T_tok == 0 || x_packed == nullptr) return err;   // no packed buffer: index only
    const int gblocks = (T_tok + 3) / 4;
    const int passes = (d / (bf16 ? 8 : 4) + kWave - 1) / kWave;
#define DICEMOE_GATHER(T_, NP_)                                                                                      \
    hipLaunchKernelGGL((dispatch_gather_kernel<T_, NP_>), dim3(gblocks), dim3(256), 0, stream, static_cast<const T_*>(x), \
                       inv, T_tok, d, k, mask == nullptr ? 1 : 0, static_cast<T_*>(x_packed))
    if (bf16) {
        if (passes == 1) DICEMOE_GATHER(bf16_t, 1);
        else if (passes == 2) DICEMOE_GATHER(bf16_t, 2);
        else if (passes == 3) DICEMOE_GATHER(bf16_t, 3);
        else if (passes == 4) DICEMOE_GATHER(bf16_t, 4);
        else DICEMOE_GATHER(bf16_t, 0);
    } else {
        if (passes == 1) DICEMOE_GATHER(float, 1);
        else if (passes == 2) DICEMOE_GATHER(float, 2);
        else if (passes <= 4) DICEMOE_GATHER(float, 4);
        else DICEMOE_GATHER(float, 0);
    }
#undef DICEMOE_GATHER
    return hipGetLastError();
}

// ---- scratch for callers that cannot hand over a workspace (moe_dispatch_noalloc)
// One array per device, held until the process ends.  Host code never uses the array's name as an
// address: the device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = 64 * 1024;
static __device__ __align__(256) int32_t scratch[kStaticScratchBytes / sizeof(int32_t)];

constexpr int kMaxDevices = 64;
static int32_t* g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each device, null until looked up
static std::mutex g_scratch_lock;

size_t dispatch_static_scratch_bytes() { return kStaticScratchBytes; }

hipError_t dispatch_static_scratch(int32_t** out)
{
    int device = -1;
    hipError_t err = hipGetDevice(&device);
    if (err != hipSuccess) return err;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (g_scratch_ptr[device] == nullptr) {
        void* ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));      // the current device's copy of the array
        if (err != hipSuccess) return err;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<int32_t*>(ptr);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
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
