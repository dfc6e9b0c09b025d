// Router kernel: logits, top-K by logit (ties to the lower expert id), softmax scores.
// Follows Algorithm 1 of the paper ("[s, idx] <- router(x)") with K activated experts per
// token (Conditional Communication figure caption).
//
// One wavefront owns one token at a time.  Each lane multiplies its 16-byte slices of the
// token's row with the matching slices of every expert's router row (staged in LDS when it
// fits), the E partial sums are reduced over the 64 lanes with a fixed butterfly, and then lane
// e plays expert e: it ranks its logit against the others and, if it is among the K largest,
// writes its index and probability.  The kernel is bound by reading x once from HBM.
#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

template <typename T, int EMAX, bool LDS_W>
__global__ __launch_bounds__(256) void gate_kernel(const T* __restrict__ x, const T* __restrict__ Wg,
                                                   const float* __restrict__ bg, int T_tok, int d, int E,
                                                   int k, int renorm, float* __restrict__ scores,
                                                   int32_t* __restrict__ expert_idx,
                                                   float* __restrict__ probs_all, float* __restrict__ logits)
{
    constexpr int V = Store<T>::kVec;
    extern __shared__ uint4 lds_w[];
    const int nvec = d / V;
    const uint4* wsrc = reinterpret_cast<const uint4*>(Wg);
    if (LDS_W) {
        for (int v = threadIdx.x; v < E * nvec; v += blockDim.x) lds_w[v] = wsrc[v];
        __syncthreads();
    }
    const uint4* wv = LDS_W ? lds_w : wsrc;
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    const int waves_per_block = blockDim.x / kWave;

    for (int tok = blockIdx.x * waves_per_block + wave; tok < T_tok; tok += gridDim.x * waves_per_block) {
        float acc[EMAX];
#pragma unroll
        for (int e = 0; e < EMAX; ++e) acc[e] = 0.f;
        const uint4* xr = reinterpret_cast<const uint4*>(x + static_cast<size_t>(tok) * d);
        for (int c = lane; c < nvec; c += kWave) {
            float xf[V];
            Store<T>::unpack(xr[c], xf);
#pragma unroll
            for (int e = 0; e < EMAX; ++e) {
                if (e < E) {
                    float wf[V];
                    Store<T>::unpack(wv[e * nvec + c], wf);
#pragma unroll
                    for (int t = 0; t < V; ++t) acc[e] = fmaf(xf[t], wf[t], acc[e]);
                }
            }
        }
        float zmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) {
                acc[e] = wave_sum(acc[e]);
                if (bg) acc[e] += bg[e];
                zmax = fmaxf(zmax, acc[e]);
            }
        }
        // lane e is expert e
        float z_me = -INFINITY;
        float denom = 0.f;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) {
                if (lane == e) z_me = acc[e];
                denom += expf(acc[e] - zmax);
            }
        }
        int rank = 0;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) rank += (acc[e] > z_me || (acc[e] == z_me && e < lane)) ? 1 : 0;
        }
        const bool is_expert = lane < E;
        const float p_me = is_expert ? expf(z_me - zmax) / denom : 0.f;
        const bool chosen = is_expert && rank < k;
        float s_me = p_me;
        if (renorm) {
            const float ssum = wave_sum(chosen ? p_me : 0.f);
            s_me = p_me / ssum;
        }
        if (chosen) {
            scores[static_cast<size_t>(tok) * k + rank] = s_me;
            expert_idx[static_cast<size_t>(tok) * k + rank] = lane;
        }
        if (is_expert) {
            if (probs_all) probs_all[static_cast<size_t>(tok) * E + lane] = p_me;
            if (logits) logits[static_cast<size_t>(tok) * E + lane] = z_me;
        }
    }
}

template <typename T, int EMAX>
static hipError_t launch_gate_e(const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                                int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                hipStream_t stream)
{
    const int waves_per_block = 4;
    int blocks = (T_tok + waves_per_block - 1) / waves_per_block;
    const int max_blocks = 256 * 4;  // a few blocks per compute unit; each wave then loops over tokens
    if (blocks > max_blocks) blocks = max_blocks;
    const size_t w_bytes = static_cast<size_t>(E) * d * sizeof(T);
    if (w_bytes <= 64 * 1024) {
        hipLaunchKernelGGL((gate_kernel<T, EMAX, true>), dim3(blocks), dim3(256), w_bytes, stream,
                           static_cast<const T*>(x), static_cast<const T*>(Wg), bg, T_tok, d, E, k, renorm,
                           scores, idx, probs, logits);
    } else {
        hipLaunchKernelGGL((gate_kernel<T, EMAX, false>), dim3(blocks), dim3(256), 0, stream,
                           static_cast<const T*>(x), static_cast<const T*>(Wg), bg, T_tok, d, E, k, renorm,
                           scores, idx, probs, logits);
    }
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_gate_t(const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                                int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                hipStream_t stream)
{
    if (E <= 8) return launch_gate_e<T, 8>(x, Wg, bg, T_tok, d, E, k, renorm, scores, idx, probs, logits, stream);
    if (E <= 16) return launch_gate_e<T, 16>(x, Wg, bg, T_tok, d, E, k, renorm, scores, idx, probs, logits, stream);
    if (E <= 32) return launch_gate_e<T, 32>(x, Wg, bg, T_tok, d, E, k, renorm, scores, idx, probs, logits, stream);
    return launch_gate_e<T, 64>(x, Wg, bg, T_tok, d, E, k, renorm, scores, idx, probs, logits, stream);
}

hipError_t launch_gate(bool bf16, const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                       int renorm, float* scores, int32_t* idx, float* probs, float* logits, hipStream_t stream)
{
    if (bf16) return launch_gate_t<bf16_t>(x, Wg, bg, T_tok, d, E, k, renorm, scores, idx, probs, logits, stream);
    return launch_gate_t<float>(x, Wg, bg, T_tok, d, E, k, renorm, scores, idx, probs, logits, stream);
}

}  // namespace dicemoe
