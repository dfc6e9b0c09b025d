// Conditional Communication decision (supplement, Algorithm 4): which (token, slot) pairs are
// recomputed this step and which reuse the cached expert output.
//
// ALL / NONE / ALG4 are elementwise.  The fraction policies need an exact top-m selection of
// tokens by a float score with ties going to the lower token index; one workgroup does it with a
// most-significant-digit radix select on the score's bit pattern (4 passes of 8 bits, LDS
// histograms), then resolves ties at the threshold by a block-wide prefix count in index order.
// Everything is integer work on the bit patterns, so the mask is reproducible bit for bit.
#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

// Counter-based draw of the "Random" ablation variant: the 32-bit avalanche step of MurmurHash3 (a
// published bit mixer) on seed * 0x9E3779B9 + token, modulo 2^32.
__device__ __forceinline__ uint32_t mix32(uint32_t seed, uint32_t token) {
    uint32_t h = seed * 0x9E3779B9u + token;
    h ^= h >> 16; h *= 0x85EBCA6Bu;
    h ^= h >> 13; h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

// kc = columns of the mask (k routed slots, then the shared-expert slots, which are always refreshed).
// kind 1 / 5 / 6: Algorithm 4 with the always-fresh slot being the top-1 slot, the last activated
// slot ("High Score" deprioritised) or a slot drawn per token ("Random"), Section 5.3 ablation.
__global__ __launch_bounds__(256) void refresh_simple_kernel(int kind, int N, int kc, int k, int off_step,
                                                             uint32_t seed, uint8_t* __restrict__ mask,
                                                             int32_t* __restrict__ n_refresh, int n_value)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p == 0) *n_refresh = n_value;
    if (p >= N) return;
    const int j = p % kc;
    uint8_t m;
    if (j >= k) m = 1;                                      // shared expert: fresh in every step
    else if (kind == 0) m = 1;                              // every pair
    else if (kind == 4) m = 0;                              // no pair
    else {
        int fresh_slot = 0;                                 // top-1 slot always, others on t mod n == 0
        if (kind == 5) fresh_slot = k - 1;
        else if (kind == 6) fresh_slot = static_cast<int>(mix32(seed, static_cast<uint32_t>(p / kc)) % static_cast<uint32_t>(k));
        m = (j == fresh_slot || !off_step) ? 1 : 0;
    }
    mask[p] = m;
}

// monotone map from float bits to unsigned: larger float <-> larger key
__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;

__global__ __launch_bounds__(kSelThreads) void refresh_select_any_kernel(const float* __restrict__ scores, int T_tok,
                                                                    int kc, int k, int slot, int m, int token_mode,
                                                                    int n_value, uint8_t* __restrict__ mask,
                                                                    int32_t* __restrict__ n_refresh)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sfx[2][256];
    __shared__ uint32_t s_prefix, s_remaining, s_equal;
    __shared__ int wave_cnt[kSelWaves];
    const int tid = threadIdx.x;
    if (tid == 0) { *n_refresh = n_value; s_prefix = 0; s_remaining = static_cast<uint32_t>(m); s_equal = 0; }

    const bool need_select = (m > 0 && m < T_tok);
    if (need_select) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix;       // both stable until the end of this pass
            const uint32_t rem = s_remaining;
            for (int i = tid; i < T_tok; i += kSelThreads) {
                const uint32_t key = order_key(scores[static_cast<size_t>(i) * kc + slot]);
                const bool in_play = (pass == 0) || ((key >> (shift + 8)) == (prefix >> (shift + 8)));
                if (in_play) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            // sfx[b] = number of in-play keys whose digit is larger than b (suffix sum, exclusive)
            int cur = 0;
            if (tid < 256) sfx[0][tid] = (tid < 255) ? hist[tid + 1] : 0u;
            __syncthreads();
            for (int step = 1; step < 256; step <<= 1) {
                if (tid < 256) {
                    uint32_t v = sfx[cur][tid];
                    if (tid + step < 256) v += sfx[cur][tid + step];
                    sfx[cur ^ 1][tid] = v;
                }
                cur ^= 1;
                __syncthreads();
            }
            if (tid < 256) {
                const uint32_t above = sfx[cur][tid];
                if (above < rem && rem <= above + hist[tid]) {   // exactly one digit satisfies this
                    s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
                    s_remaining = rem - above;
                    s_equal = hist[tid];            // after the last pass: the keys equal to the threshold
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    const uint32_t thr = s_prefix;
    const int admit_equal = static_cast<int>(s_remaining);  // keys equal to thr to admit, in index order
    // every key equal to the threshold is admitted (no tie straddles the cut, the usual case): no ordering needed
    const bool all_equal_in = need_select && admit_equal == static_cast<int>(s_equal);
    const int wave = tid / kWave;
    int running = 0;
    for (int base = 0; base < T_tok; base += kSelThreads) {
        const int i = base + tid;
        const bool valid = i < T_tok;
        bool sel;
        if (!need_select) {
            sel = (m > 0);
        } else if (all_equal_in) {
            sel = valid && order_key(scores[static_cast<size_t>(i) * kc + slot]) >= thr;
        } else {
            const uint32_t key = valid ? order_key(scores[static_cast<size_t>(i) * kc + slot]) : 0u;
            const bool eq = valid && key == thr;
            const uint64_t b = __ballot(eq);
            if (lane_id() == 0) wave_cnt[wave] = __popcll(b);
            __syncthreads();
            int before = running + __popcll(b & lanemask_lt());
            int total = 0;
            for (int w = 0; w < kSelWaves; ++w) {
                const int c = wave_cnt[w];
                if (w < wave) before += c;
                total += c;
            }
            running += total;
            sel = valid && (key > thr || (eq && before < admit_equal));
            __syncthreads();
        }
        if (valid) {
            for (int j = 0; j < kc; ++j) {
                uint8_t v;
                if (j >= k) v = 1;                                   // shared expert: fresh in every step
                else if (token_mode) v = sel ? 1 : 0;
                else v = (j < slot) ? 1 : (j == slot ? (sel ? 1 : 0) : 0);
                mask[static_cast<size_t>(i) * kc + j] = v;
            }
        }
    }
}

// The same selection for up to 16 * 1024 tokens, keys held in registers (KPT per thread, token
// i = u * 1024 + tid).  A most-significant-digit radix select on (key - smallest key): the digit is the
// top 11 bits of the span the keys still in play cover, so that the 2048 counters are spread over the
// keys' real range (router scores share their sign and most of their exponent bits: fixed bit fields
// would send every key to two or three counters, and LDS atomics on one address serialise).  Round r
// narrows the span by 2^11; it ends early when every key of the threshold digit is admitted, which is
// the usual case after the second round.  Ties at the threshold go to the lower token, by a block-wide
// prefix count in token order.
constexpr int kSelBins = 2048;

template <int KPT>
__global__ __launch_bounds__(kSelThreads) void refresh_select_kernel(const float* __restrict__ scores, int T_tok,
                                                                    int kc, int k, int slot, int m, int token_mode,
                                                                    int n_value, uint8_t* __restrict__ mask,
                                                                    int32_t* __restrict__ n_refresh)
{
    __shared__ uint32_t hist[kSelBins];
    __shared__ uint32_t wave_a[kSelWaves], wave_b[kSelWaves];
    __shared__ uint32_t s_bin, s_above, s_cnt;
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = lane_id();
    if (tid == 0) *n_refresh = n_value;

    uint32_t key[KPT];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
        const int i = u * kSelThreads + tid;
        key[u] = order_key(scores[static_cast<size_t>(i < T_tok ? i : T_tok - 1) * kc + slot]);
    }
    const bool need_select = (m > 0 && m < T_tok);
    uint32_t lo = 0, thr = 0;
    int admit_equal = 0;          // > 0: keys equal to thr are admitted in token order, this many of them
    bool ties = false;
    if (need_select) {
        // smallest and largest key
        uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
        for (int u = 0; u < KPT; ++u)
            if (u * kSelThreads + tid < T_tok) { kmin = key[u] < kmin ? key[u] : kmin; kmax = key[u] > kmax ? key[u] : kmax; }
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) {
            const uint32_t a = __shfl_xor(kmin, sh, kWave), b = __shfl_xor(kmax, sh, kWave);
            kmin = a < kmin ? a : kmin;
            kmax = b > kmax ? b : kmax;
        }
        if (lane == 0) { wave_a[wave] = kmin; wave_b[wave] = kmax; }
        __syncthreads();
        kmin = wave_a[lane & (kSelWaves - 1)];
        kmax = wave_b[lane & (kSelWaves - 1)];
#pragma unroll
        for (int sh = kSelWaves / 2; sh >= 1; sh >>= 1) {
            const uint32_t a = __shfl_xor(kmin, sh, kWave), b = __shfl_xor(kmax, sh, kWave);
            kmin = a < kmin ? a : kmin;
            kmax = b > kmax ? b : kmax;
        }
        lo = kmin;
        uint32_t span = kmax - kmin;              // keys in play lie in [lo, lo + span]
        uint32_t remaining = static_cast<uint32_t>(m);
        for (;;) {
            const int shift = span >= kSelBins ? (32 - __builtin_clz(span)) - 11 : 0;     // span >> shift < 2048
            __syncthreads();                      // the previous round's reads of hist / s_* are done
            hist[tid] = 0; hist[tid + kSelThreads] = 0;
            __syncthreads();
#pragma unroll
            for (int u = 0; u < KPT; ++u) {
                const uint32_t rel = key[u] - lo;
                if (u * kSelThreads + tid < T_tok && key[u] >= lo && rel <= span) atomicAdd(&hist[rel >> shift], 1u);
            }
            __syncthreads();
            // keys in digits above each digit: thread t owns digits 2t and 2t+1; suffix sums over the
            // threads of a wave by shuffles, over the waves through LDS
            const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
            uint32_t incl = h0 + h1;              // becomes the sum over lanes >= this one
#pragma unroll
            for (int sh = 1; sh < kWave; sh <<= 1) {
                const uint32_t v = __shfl_down(incl, sh, kWave);
                if (lane + sh < kWave) incl += v;
            }
            if (lane == 0) wave_a[wave] = incl;
            __syncthreads();
            uint32_t higher = 0;
#pragma unroll
            for (int w = 0; w < kSelWaves; ++w) higher += (w > wave) ? wave_a[w] : 0u;
            const uint32_t above1 = higher + incl - (h0 + h1);     // keys in digits above 2t+1
            const uint32_t above0 = above1 + h1;                    // keys in digits above 2t
            if (above1 < remaining && remaining <= above1 + h1) { s_bin = 2 * tid + 1; s_above = above1; s_cnt = h1; }
            if (above0 < remaining && remaining <= above0 + h0) { s_bin = 2 * tid; s_above = above0; s_cnt = h0; }
            __syncthreads();
            const uint32_t bin = s_bin, cnt = s_cnt;
            remaining -= s_above;
            lo += bin << shift;
            if (remaining == cnt) { thr = lo; break; }              // the whole digit is admitted: keys >= lo
            if (shift == 0) { thr = lo; ties = true; admit_equal = static_cast<int>(remaining); break; }
            span = (1u << shift) - 1u;
        }
    }

    int running = 0;
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
        const int i = u * kSelThreads + tid;
        const bool valid = i < T_tok;
        bool sel;
        if (!need_select) {
            sel = (m > 0);
        } else if (!ties) {
            sel = key[u] >= thr;
        } else {
            const bool eq = valid && key[u] == thr;
            const uint64_t b = __ballot(eq);
            __syncthreads();
            if (lane == 0) wave_a[wave] = __popcll(b);
            __syncthreads();
            int before = running + __popcll(b & lanemask_lt());
            int total = 0;
#pragma unroll
            for (int w = 0; w < kSelWaves; ++w) {
                const int c = static_cast<int>(wave_a[w]);
                if (w < wave) before += c;
                total += c;
            }
            running += total;
            sel = key[u] > thr || (eq && before < admit_equal);
        }
        if (valid) {
            for (int j = 0; j < kc; ++j) {
                uint8_t v;
                if (j >= k) v = 1;                                   // shared expert: fresh in every step
                else if (token_mode) v = sel ? 1 : 0;
                else v = (j < slot) ? 1 : (j == slot ? (sel ? 1 : 0) : 0);
                mask[static_cast<size_t>(i) * kc + j] = v;
            }
        }
    }
}

hipError_t launch_refresh_simple(int kind, int T_tok, int k, int n_shared, int off_step, uint32_t seed, int n_value,
                                 uint8_t* mask, int32_t* n_refresh, hipStream_t stream)
{
    const int kc = k + n_shared;
    const int N = T_tok * kc;
    const int blocks = N > 0 ? (N + 255) / 256 : 1;
    hipLaunchKernelGGL(refresh_simple_kernel, dim3(blocks), dim3(256), 0, stream, kind, N, kc, k, off_step, seed,
                       mask, n_refresh, n_value);
    return hipGetLastError();
}

hipError_t launch_refresh_select(const float* scores, int T_tok, int k, int n_shared, int slot, int m,
                                 bool token_mode, int n_value, uint8_t* mask, int32_t* n_refresh,
                                 hipStream_t stream)
{
    const int kc = k + n_shared, tm = token_mode ? 1 : 0;
#define DICEMOE_SELECT(KPT_)                                                                                        \
    hipLaunchKernelGGL(refresh_select_kernel<KPT_>, dim3(1), dim3(kSelThreads), 0, stream, scores, T_tok, kc, k, slot, \
                       m, tm, n_value, mask, n_refresh)
    if (T_tok < 1 || T_tok > 16 * kSelThreads)      // any size: keys re-read from memory in every round
        hipLaunchKernelGGL(refresh_select_any_kernel, dim3(1), dim3(kSelThreads), 0, stream, scores, T_tok, kc, k,
                           slot, m, tm, n_value, mask, n_refresh);
    else if (T_tok <= kSelThreads) DICEMOE_SELECT(1);
    else if (T_tok <= 2 * kSelThreads) DICEMOE_SELECT(2);
    else if (T_tok <= 4 * kSelThreads) DICEMOE_SELECT(4);
    else if (T_tok <= 8 * kSelThreads) DICEMOE_SELECT(8);
    else DICEMOE_SELECT(16);
#undef DICEMOE_SELECT
    return hipGetLastError();
}

}  // namespace dicemoe
