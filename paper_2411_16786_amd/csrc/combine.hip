// Combine + scale + cache blend: y_i = sum_j s*_ij h*_ij  (Section 4.3; Algorithm 1,
// "x_c <- all2all_combine(x_e)", "x <- scale(x_c, s)"), where a pair that Conditional
// Communication did not refresh reuses its cached expert output (Algorithm 4, "reuse stale h")
// scaled by the cached score (supplement, "Expert Score Scaling") or by this step's score.
//
// One wavefront per token gathers its k rows (fresh rows from the packed buffer through inv,
// reused rows from the cache), accumulates in float in slot order 0..k-1 (fixed order, no
// atomics: reproducible), stores y, and writes refreshed rows and scores through to the cache.
// Bound by HBM traffic: k rows read, one row written, plus the write-through.  Without a packed
// buffer (h_packed null) the expert call has already scattered the fresh rows into the cache: every
// row is then read from the cache and only the scores are written through.
#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

// KK > 0: k == KK, the per-pair scalars (packed row, score, fresh or reused) are read once per token
// and the k row loads of a 16-byte column slice are issued together; KK == 0: any k, pair by pair.
// NP > 0: a row is at most NP passes of 64 lanes x 16 bytes, and the loads of all passes are issued
// before the first result is formed (one memory round trip per token instead of one per pass: with
// sixteen wavefronts per compute unit the kernel is bound by latency, not by issue); NP == 0: any d.
// Slots k_cached..k-1 (shared experts, fresh in every step) are never written to the caches.
template <typename T, int KK, int NP>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ h_packed, const int32_t* __restrict__ inv,
                                                      const float* __restrict__ scores,
                                                      const uint8_t* __restrict__ mask, int T_tok, int d, int k,
                                                      int k_cached, T* H_cache, float* S_cache, int use_fresh,
                                                      T* __restrict__ y)
{
    constexpr int V = Store<T>::kVec;
    const int tok = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tok >= T_tok) return;
    const int lane = lane_id();
    const int nvec = d / V;
    const size_t p0 = static_cast<size_t>(tok) * k;
    const u32x4_t* hp = reinterpret_cast<const u32x4_t*>(h_packed);
    u32x4_t* hc = reinterpret_cast<u32x4_t*>(H_cache);
    u32x4_t* yo = reinterpret_cast<u32x4_t*>(y) + static_cast<size_t>(tok) * nvec;

    if (KK > 0) {
        constexpr int KN = KK > 0 ? KK : 1;
        const u32x4_t* src[KN];        // row to read for slot j, nullptr for a refreshed pair without a packed row
        float sc[KN];
        bool fresh[KN];
#pragma unroll
        for (int j = 0; j < KN; ++j) {
            const size_t p = p0 + j;
            fresh[j] = (mask == nullptr) || mask[p] != 0;
            if (fresh[j]) {
                if (hp != nullptr) {
                    const int r = inv[p];
                    src[j] = r >= 0 ? hp + static_cast<size_t>(r) * nvec : nullptr;
                } else {
                    src[j] = hc + p * nvec;            // the expert call has put the fresh row into the cache itself
                }
                sc[j] = scores[p];
            } else {
                src[j] = hc + p * nvec;
                sc[j] = use_fresh ? scores[p] : S_cache[p];
            }
        }
        if (NP > 0) {
            constexpr int NPN = NP > 0 ? NP : 1;
            u32x4_t v[NPN][KN];
#pragma unroll
            for (int p = 0; p < NPN; ++p) {
                const int c = lane + p * kWave;
#pragma unroll
                for (int j = 0; j < KN; ++j) v[p][j] = (src[j] && c < nvec) ? src[j][c] : u32x4_t{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int p = 0; p < NPN; ++p) {
                const int c = lane + p * kWave;
                if (c >= nvec) break;
                float acc[V];
#pragma unroll
                for (int t = 0; t < V; ++t) acc[t] = 0.f;
#pragma unroll
                for (int j = 0; j < KN; ++j) {
                    float f[V];
                    Store<T>::unpack(v[p][j], f);
#pragma unroll
                    for (int t = 0; t < V; ++t) acc[t] = fmaf(sc[j], f[t], acc[t]);
                    if (fresh[j] && hc && hp && j < k_cached) hc[(p0 + j) * nvec + c] = v[p][j];
                }
                const uint4 packed = Store<T>::pack(acc);
                yo[c] = u32x4_t{packed.x, packed.y, packed.z, packed.w};
            }
        } else
        for (int c = lane; c < nvec; c += kWave) {
            u32x4_t v[KN];
#pragma unroll
            for (int j = 0; j < KN; ++j) v[j] = src[j] ? src[j][c] : u32x4_t{0u, 0u, 0u, 0u};
            float acc[V];
#pragma unroll
            for (int t = 0; t < V; ++t) acc[t] = 0.f;
#pragma unroll
            for (int j = 0; j < KN; ++j) {
                float f[V];
                Store<T>::unpack(v[j], f);
#pragma unroll
                for (int t = 0; t < V; ++t) acc[t] = fmaf(sc[j], f[t], acc[t]);
                if (fresh[j] && hc && hp && j < k_cached) hc[(p0 + j) * nvec + c] = v[j];
            }
            const uint4 packed = Store<T>::pack(acc);
            yo[c] = u32x4_t{packed.x, packed.y, packed.z, packed.w};
        }
    } else {
        for (int c = lane; c < nvec; c += kWave) {
            float acc[V];
#pragma unroll
            for (int t = 0; t < V; ++t) acc[t] = 0.f;
            for (int j = 0; j < k; ++j) {
                const size_t p = p0 + j;
                const bool is_fresh = (mask == nullptr) || mask[p] != 0;
                u32x4_t v = u32x4_t{0u, 0u, 0u, 0u};
                float s;
                if (is_fresh) {
                    if (hp != nullptr) {
                        const int r = inv[p];
                        if (r >= 0) v = hp[static_cast<size_t>(r) * nvec + c];
                        if (hc && j < k_cached) hc[p * nvec + c] = v;
                    } else {
                        v = hc[p * nvec + c];
                    }
                    s = scores[p];
                } else {
                    v = hc[p * nvec + c];
                    s = use_fresh ? scores[p] : S_cache[p];
                }
                float f[V];
                Store<T>::unpack(v, f);
#pragma unroll
                for (int t = 0; t < V; ++t) acc[t] = fmaf(s, f[t], acc[t]);
            }
            const uint4 packed = Store<T>::pack(acc);
            yo[c] = u32x4_t{packed.x, packed.y, packed.z, packed.w};
        }
    }
    if (S_cache && lane < k_cached) {
        const size_t p = p0 + lane;
        if (mask == nullptr || mask[p] != 0) S_cache[p] = scores[p];
    }
}

template <typename T>
static void launch_combine_t(const void* h_packed, const int32_t* inv, const float* scores, const uint8_t* mask,
                             int T_tok, int d, int k, int k_cached, void* H_cache, float* S_cache, int use_fresh,
                             void* y, hipStream_t stream)
{
    const int blocks = (T_tok + 3) / 4;
    const int passes = (d / Store<T>::kVec + kWave - 1) / kWave;
#define DICEMOE_COMBINE_NP(KK_, NP_)                                                                                  \
    hipLaunchKernelGGL((combine_kernel<T, KK_, NP_>), dim3(blocks), dim3(256), 0, stream, static_cast<const T*>(h_packed), \
                       inv, scores, mask, T_tok, d, k, k_cached, static_cast<T*>(H_cache), S_cache, use_fresh,             \
                       static_cast<T*>(y))
#define DICEMOE_COMBINE(KK_)                                                  \
    do {                                                                      \
        if (passes == 1) DICEMOE_COMBINE_NP(KK_, 1);                          \
        else if (passes == 2) DICEMOE_COMBINE_NP(KK_, 2);                     \
        else if (passes == 3) DICEMOE_COMBINE_NP(KK_, 3);                     \
        else if (passes == 4) DICEMOE_COMBINE_NP(KK_, 4);                     \
        else DICEMOE_COMBINE_NP(KK_, 0);                                      \
    } while (0)
    if (k == 1) DICEMOE_COMBINE(1);
    else if (k == 2) DICEMOE_COMBINE(2);
    else if (k == 3) DICEMOE_COMBINE(3);
    else if (k == 4) DICEMOE_COMBINE(4);
    else DICEMOE_COMBINE_NP(0, 0);
#undef DICEMOE_COMBINE_NP
#undef DICEMOE_COMBINE
}

hipError_t launch_combine(bool bf16, const void* h_packed, const int32_t* inv, const float* scores,
                          const uint8_t* mask, int T_tok, int d, int k, int k_cached, void* H_cache,
                          float* S_cache, int use_fresh, void* y, hipStream_t stream)
{
    if (T_tok == 0) return hipSuccess;
    if (bf16) launch_combine_t<bf16_t>(h_packed, inv, scores, mask, T_tok, d, k, k_cached, H_cache, S_cache, use_fresh, y, stream);
    else launch_combine_t<float>(h_packed, inv, scores, mask, T_tok, d, k, k_cached, H_cache, S_cache, use_fresh, y, stream);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void commit_scores_kernel(const float* __restrict__ scores,
                                                           const uint8_t* __restrict__ mask, int n_pairs, int k,
                                                           int k_cached, float* __restrict__ S_buffer)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pairs || p % k >= k_cached) return;
    if (mask == nullptr || mask[p] != 0) S_buffer[p] = scores[p];
}

hipError_t launch_commit_scores(const float* scores, const uint8_t* mask, int T_tok, int k, int k_cached,
                                float* S_buffer, hipStream_t stream)
{
    const int n_pairs = T_tok * k;
    if (n_pairs == 0) return hipSuccess;
    hipLaunchKernelGGL(commit_scores_kernel, dim3((n_pairs + 255) / 256), dim3(256), 0, stream, scores, mask, n_pairs, k,
                       k_cached, S_buffer);
    return hipGetLastError();
}

}  // namespace dicemoe
