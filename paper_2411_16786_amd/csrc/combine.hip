// Combine + scale + cache blend: y_i = sum_j s*_ij h*_ij  (Section 4.3; Algorithm 1,
// "x_c <- all2all_combine(x_e)", "x <- scale(x_c, s)"), where a pair that Conditional
// Communication did not refresh reuses its cached expert output (Algorithm 4, "reuse stale h")
// scaled by the cached score (supplement, "Expert Score Scaling") or by this step's score.
//
// One wavefront per token gathers its k rows (fresh rows from the packed buffer through inv,
// reused rows from the cache), accumulates in float in slot order 0..k-1 (fixed order, no
// atomics: reproducible), stores y, and writes refreshed rows and scores through to the cache.
// Bound by HBM traffic: k rows read, one row written, plus the write-through.
#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ h_packed, const int32_t* __restrict__ inv,
                                                      const float* __restrict__ scores,
                                                      const uint8_t* __restrict__ mask, int T_tok, int d, int k,
                                                      T* H_cache, float* S_cache, int use_fresh, T* __restrict__ y)
{
    constexpr int V = Store<T>::kVec;
    const int tok = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (tok >= T_tok) return;
    const int lane = lane_id();
    const int nvec = d / V;
    const size_t p0 = static_cast<size_t>(tok) * k;
    const uint4* hp = reinterpret_cast<const uint4*>(h_packed);
    uint4* hc = reinterpret_cast<uint4*>(H_cache);
    uint4* yo = reinterpret_cast<uint4*>(y) + static_cast<size_t>(tok) * nvec;

    for (int c = lane; c < nvec; c += kWave) {
        float acc[V];
#pragma unroll
        for (int t = 0; t < V; ++t) acc[t] = 0.f;
        for (int j = 0; j < k; ++j) {
            const size_t p = p0 + j;
            const bool fresh = (mask == nullptr) || mask[p] != 0;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            float s;
            if (fresh) {
                const int r = inv[p];
                if (r >= 0) v = hp[static_cast<size_t>(r) * nvec + c];
                s = scores[p];
                if (hc) hc[p * nvec + c] = v;
            } else {
                v = hc[p * nvec + c];
                s = use_fresh ? scores[p] : S_cache[p];
            }
            float f[V];
            Store<T>::unpack(v, f);
#pragma unroll
            for (int t = 0; t < V; ++t) acc[t] = fmaf(s, f[t], acc[t]);
        }
        yo[c] = Store<T>::pack(acc);
    }
    if (S_cache && lane < k) {
        const size_t p = p0 + lane;
        if (mask == nullptr || mask[p] != 0) S_cache[p] = scores[p];
    }
}

hipError_t launch_combine(bool bf16, const void* h_packed, const int32_t* inv, const float* scores,
                          const uint8_t* mask, int T_tok, int d, int k, void* H_cache, float* S_cache,
                          int use_fresh, void* y, hipStream_t stream)
{
    if (T_tok == 0) return hipSuccess;
    const int blocks = (T_tok + 3) / 4;
    if (bf16)
        hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(blocks), dim3(256), 0, stream,
                           static_cast<const bf16_t*>(h_packed), inv, scores, mask, T_tok, d, k,
                           static_cast<bf16_t*>(H_cache), S_cache, use_fresh, static_cast<bf16_t*>(y));
    else
        hipLaunchKernelGGL(combine_kernel<float>, dim3(blocks), dim3(256), 0, stream,
                           static_cast<const float*>(h_packed), inv, scores, mask, T_tok, d, k,
                           static_cast<float*>(H_cache), S_cache, use_fresh, static_cast<float*>(y));
    return hipGetLastError();
}

}  // namespace dicemoe
