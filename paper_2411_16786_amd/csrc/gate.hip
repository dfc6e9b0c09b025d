// Router kernel: logits, top-K by logit (ties to the lower expert id), softmax scores.
// Follows Algorithm 1 of the paper ("[s, idx] <- router(x)") with K activated experts per
// token (Conditional Communication figure caption).
//
// bf16 storage: gate_mfma_kernel (below) puts the skinny GEMM on the matrix cores.
// float storage (small workloads): gate_kernel.  One wavefront owns TPW tokens at a time.  Each lane first issues the loads of its 16-byte slices
// of all TPW rows (NCH slices per row; they are in flight while the workgroup stages the router
// matrix in LDS), multiplies them with the matching slices of every expert's router row, and the
// E x TPW partial sums are reduced over the 64 lanes with a fixed butterfly.  Then lane e plays
// expert e: it ranks its logit against the others and, if it is among the K largest, writes its
// index and probability.  The kernel is bound by reading x once from HBM.
#include <type_traits>
#include "common.hpp"
#include "kernels.hpp"

namespace dicemoe {

template <typename T, int EMAX, int NCH, int TPW, bool LDS_W>
__global__ __launch_bounds__(256) void gate_kernel(const T* __restrict__ x, const T* __restrict__ Wg,
                                                   const float* __restrict__ bg, int T_tok, int d, int E,
                                                   int k, int n_shared, int renorm, float* __restrict__ scores,
                                                   int32_t* __restrict__ expert_idx,
                                                   float* __restrict__ probs_all, float* __restrict__ logits)
{
    constexpr int V = Store<T>::kVec;
    extern __shared__ u32x4_t lds_w[];
    const int nvec = d / V;
    const u32x4_t* wsrc = reinterpret_cast<const u32x4_t*>(Wg);
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    const int tok0 = (blockIdx.x * (blockDim.x / kWave) + wave) * TPW;

    // this lane's slices of the TPW rows (rows past the end repeat the last token; never written)
    u32x4_t xv[TPW][NCH];
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        int tok = tok0 + t;
        if (tok >= T_tok) tok = T_tok - 1;
        const u32x4_t* xr = reinterpret_cast<const u32x4_t*>(x + static_cast<size_t>(tok) * d);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int i = lane + c * kWave;
            xv[t][c] = xr[i < nvec ? i : 0];
        }
    }
    if (LDS_W) {
        for (int v = threadIdx.x; v < E * nvec; v += blockDim.x) lds_w[v] = wsrc[v];
        __syncthreads();
    }
    if (tok0 >= T_tok) return;
    const u32x4_t* wv = LDS_W ? lds_w : wsrc;

    float acc[TPW][EMAX];
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int e = 0; e < EMAX; ++e) acc[t][e] = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int i = lane + c * kWave;
        if (i < nvec) {
            float xf[TPW][V];
#pragma unroll
            for (int t = 0; t < TPW; ++t) Store<T>::unpack(xv[t][c], xf[t]);
#pragma unroll
            for (int e = 0; e < EMAX; ++e) {
                if (e < E) {
                    float wf[V];
                    Store<T>::unpack(wv[e * nvec + i], wf);
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
#pragma unroll
                        for (int u = 0; u < V; ++u) acc[t][e] = fmaf(xf[t][u], wf[u], acc[t][e]);
                }
            }
        }
    }

#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int tok = tok0 + t;
        float zmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) {
                acc[t][e] = wave_sum(acc[t][e]);
                if (bg) acc[t][e] += bg[e];
                zmax = fmaxf(zmax, acc[t][e]);
            }
        }
        // lane e is expert e
        float z_me = -INFINITY;
        float denom = 0.f;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) {
                if (lane == e) z_me = acc[t][e];
                denom += expf(acc[t][e] - zmax);
            }
        }
        int rank = 0;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) rank += (acc[t][e] > z_me || (acc[t][e] == z_me && e < lane)) ? 1 : 0;
        }
        const bool is_expert = lane < E;
        const float p_me = is_expert ? expf(z_me - zmax) / denom : 0.f;
        const bool chosen = is_expert && rank < k;
        float s_me = p_me;
        if (renorm) {
            const float ssum = wave_sum(chosen ? p_me : 0.f);
            s_me = p_me / ssum;
        }
        if (tok < T_tok) {
            const size_t row = static_cast<size_t>(tok) * (k + n_shared);
            if (chosen) {
                scores[row + rank] = s_me;
                expert_idx[row + rank] = lane;
            }
            if (lane < n_shared) {                      // shared experts: every token, score 1
                scores[row + k + lane] = 1.0f;
                expert_idx[row + k + lane] = E + lane;
            }
            if (is_expert) {
                if (probs_all) probs_all[static_cast<size_t>(tok) * E + lane] = p_me;
                if (logits) logits[static_cast<size_t>(tok) * E + lane] = z_me;
            }
        }
    }
}

// A value of the lane N places away inside the caller's row of 16 lanes (DPP row rotation; N = 1 .. 15
// visits every other lane of the row once).
template <int N>
__device__ __forceinline__ int row_rotate(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x120 + N, 0xF, 0xF, true);
}
template <int N>
__device__ __forceinline__ float row_rotate(float v) {
    return __builtin_bit_cast(float, row_rotate<N>(__builtin_bit_cast(int, v)));
}
template <int N, typename F>
__device__ __forceinline__ void for_row_rotations(F&& f) {
    if constexpr (N < 16) {
        f(std::integral_constant<int, N>{});
        for_row_rotations<N + 1>(f);
    }
}

// bf16 router on the matrix cores.  A workgroup owns 16 tokens; logits[16][E] = x[16][d] . Wg[E][d]^T
// is a chain of v_mfma_f32_16x16x32_bf16 steps over k, split round robin over the 4 wavefronts
// (wavefront w takes k-steps w, w+4, ...).  Operands come straight from global memory in MFMA
// layout: lane l supplies row l%16 (a token for x, an expert for Wg) and the 8 consecutive k
// values 8*(l/16).. of the step, i.e. one 16-byte load each; all loads of a batch are issued before
// its MFMAs.  Accumulator register v of lane l is logits[token 4*(l/16)+v][expert l%16].  The four
// partial sums meet in LDS and are added in wavefront order (fixed, reproducible).  With at most 16
// experts thread (t, e) then finishes logit e of token t: the 16 lanes of a DPP row hold one token and
// rank, maximum and softmax sum come from rotating the row (no further LDS trip, all 16 tokens at once);
// with more experts wavefront w finishes tokens 4w..4w+3 with lane e playing expert e.  Rank is by
// logit, ties to the lower id.
// U = k-steps per batch and wavefront: the launcher picks it so that one batch covers a wavefront's
// whole share of the row (a single round trip to memory) whenever that fits in registers.
template <int NB, int U>
__global__ __launch_bounds__(256) void gate_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wg,
                                                        const float* __restrict__ bg, int T_tok, int d, int E,
                                                        int k, int n_shared, int renorm, float* __restrict__ scores,
                                                        int32_t* __restrict__ expert_idx,
                                                        float* __restrict__ probs_all, float* __restrict__ logits)
{
    typedef __bf16 bf16x8_g __attribute__((ext_vector_type(8)));
    typedef float f32x4_g __attribute__((ext_vector_type(4)));
    constexpr int EP = NB * 16;                  // padded expert count
    __shared__ float part[4][16][EP];
    __shared__ float zfin[16][EP];
    const int wave = threadIdx.x / kWave;
    const int lane = lane_id();
    const int row = lane & 15, kq = lane >> 4;
    const int tok0 = blockIdx.x * 16;
    int tok = tok0 + row;
    if (tok >= T_tok) tok = T_tok - 1;           // rows past the end repeat the last token; never written
    const u32x4_t* xa = reinterpret_cast<const u32x4_t*>(x + static_cast<size_t>(tok) * d);
    const u32x4_t* wb[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int e = nb * 16 + row;
        if (e >= E) e = E - 1;                   // padding columns repeat the last expert; ignored later
        wb[nb] = reinterpret_cast<const u32x4_t*>(Wg + static_cast<size_t>(e) * d);
    }
    f32x4_g acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_g{0.f, 0.f, 0.f, 0.f};

    const int nsteps = d / 32;
    for (int s0 = wave; s0 < nsteps; s0 += 4 * U) {
        u32x4_t av[U], bv[NB][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int sidx = s0 + 4 * u;
            const bool on = sidx < nsteps;
            const int unit = (on ? sidx : s0) * 4 + kq;
            av[u] = xa[unit];
            if (!on) av[u] = u32x4_t{0u, 0u, 0u, 0u};      // a step past the end contributes zero
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) bv[nb][u] = wb[nb][unit];
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_g*>(&av[u]),
                                                                  *reinterpret_cast<const bf16x8_g*>(&bv[nb][u]),
                                                                  acc[nb], 0, 0, 0);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 4; ++v) part[wave][4 * kq + v][nb * 16 + row] = acc[nb][v];
    __syncthreads();
    if (NB == 1) {
        // Up to 16 experts: thread (t, e) = (tid / 16, tid % 16) finishes logit e of token t, so a row of 16
        // lanes is one token and every lane meets the 15 other logits of its token by rotating the row.
        const int t = threadIdx.x >> 4, e = threadIdx.x & 15;
        const bool is_expert = e < E;
        float z = ((part[0][t][e] + part[1][t][e]) + part[2][t][e]) + part[3][t][e];   // wavefront order, then the bias
        if (bg && is_expert) z += bg[e];
        const float z_me = is_expert ? z : -INFINITY;       // padding lanes never outrank an expert
        float zmax = z_me;
        int rank = 0;
        for_row_rotations<1>([&](auto n) {
            const float z_o = row_rotate<decltype(n)::value>(z_me);
            const int e_o = row_rotate<decltype(n)::value>(e);
            zmax = fmaxf(zmax, z_o);
            rank += (z_o > z_me || (z_o == z_me && e_o < e)) ? 1 : 0;
        });
        const float q_me = is_expert ? expf(z_me - zmax) : 0.f;
        float denom = q_me;
        for_row_rotations<1>([&](auto n) { denom += row_rotate<decltype(n)::value>(q_me); });
        const float p_me = q_me / denom;
        const bool chosen = is_expert && rank < k;
        float s_me = p_me;
        if (renorm) {
            const float c_me = chosen ? p_me : 0.f;
            float ssum = c_me;
            for_row_rotations<1>([&](auto n) { ssum += row_rotate<decltype(n)::value>(c_me); });
            s_me = p_me / ssum;
        }
        const int tk = tok0 + t;
        if (tk < T_tok) {
            const size_t row = static_cast<size_t>(tk) * (k + n_shared);
            if (chosen) {
                scores[row + rank] = s_me;
                expert_idx[row + rank] = e;
            }
            for (int sh = e; sh < n_shared; sh += 16) {     // shared experts: every token, score 1
                scores[row + k + sh] = 1.0f;
                expert_idx[row + k + sh] = E + sh;
            }
            if (is_expert) {
                if (probs_all) probs_all[static_cast<size_t>(tk) * E + e] = p_me;
                if (logits) logits[static_cast<size_t>(tk) * E + e] = z_me;
            }
        }
        return;
    }
    // logits: the four partial sums in wavefront order, then the bias
    for (int i = threadIdx.x; i < 16 * EP; i += blockDim.x) {
        const int t = i / EP, e = i % EP;
        float z = ((part[0][t][e] + part[1][t][e]) + part[2][t][e]) + part[3][t][e];
        if (bg && e < E) z += bg[e];
        zfin[t][e] = z;
    }
    __syncthreads();

    for (int tt = 0; tt < 4; ++tt) {
        const int t = wave * 4 + tt;
        const int tk = tok0 + t;
        if (tk >= T_tok) break;                  // uniform across the wavefront
        const bool is_expert = lane < E;
        const float z_me = is_expert ? zfin[t][lane] : -INFINITY;
        float zmax = -INFINITY;
        for (int e = 0; e < E; ++e) zmax = fmaxf(zmax, zfin[t][e]);
        float denom = 0.f;
        int rank = 0;
        for (int e = 0; e < E; ++e) {
            const float z = zfin[t][e];
            denom += expf(z - zmax);
            rank += (z > z_me || (z == z_me && e < lane)) ? 1 : 0;
        }
        const float p_me = is_expert ? expf(z_me - zmax) / denom : 0.f;
        const bool chosen = is_expert && rank < k;
        float s_me = p_me;
        if (renorm) {
            const float ssum = wave_sum(chosen ? p_me : 0.f);
            s_me = p_me / ssum;
        }
        const size_t row = static_cast<size_t>(tk) * (k + n_shared);
        if (chosen) {
            scores[row + rank] = s_me;
            expert_idx[row + rank] = lane;
        }
        if (lane < n_shared) {                          // shared experts: every token, score 1
            scores[row + k + lane] = 1.0f;
            expert_idx[row + k + lane] = E + lane;
        }
        if (is_expert) {
            if (probs_all) probs_all[static_cast<size_t>(tk) * E + lane] = p_me;
            if (logits) logits[static_cast<size_t>(tk) * E + lane] = z_me;
        }
    }
}

template <int NB>
static hipError_t launch_gate_mfma_nb(const bf16_t* xb, const bf16_t* wb, const float* bg, int T_tok, int d, int E, int k,
                                      int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                      hipStream_t stream)
{
    const int blocks = (T_tok + 15) / 16;
    const int need = (d / 32 + 3) / 4;           // k-steps per wavefront
    // registers per lane: 4 * U * (1 + NB) for the operands of a batch
    constexpr int UMAX = NB == 1 ? 16 : (NB == 2 ? 10 : 6);
#define DICEMOE_GATE_U(U_)                                                                                          \
    if (need <= U_ || U_ == UMAX) {                                                                                 \
        hipLaunchKernelGGL((gate_mfma_kernel<NB, U_>), dim3(blocks), dim3(256), 0, stream, xb, wb, bg, T_tok, d, E, \
                           k, n_shared, renorm, scores, idx, probs, logits);                                                  \
        return hipGetLastError();                                                                                   \
    }
    DICEMOE_GATE_U(3)
    DICEMOE_GATE_U(6)
    if (UMAX >= 9) { DICEMOE_GATE_U((UMAX >= 9 ? 9 : UMAX)) }
    if (UMAX >= 10) { DICEMOE_GATE_U((UMAX >= 10 ? 10 : UMAX)) }
    if (UMAX >= 12) { DICEMOE_GATE_U((UMAX >= 12 ? 12 : UMAX)) }
    if (UMAX >= 16) { DICEMOE_GATE_U((UMAX >= 16 ? 16 : UMAX)) }
#undef DICEMOE_GATE_U
    return hipErrorInvalidValue;                 // not reached: the last case of every NB takes any d
}

static hipError_t launch_gate_mfma(const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                                   int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                   hipStream_t stream)
{
    const bf16_t* xb = static_cast<const bf16_t*>(x);
    const bf16_t* wb = static_cast<const bf16_t*>(Wg);
    if (E <= 16) return launch_gate_mfma_nb<1>(xb, wb, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream);
    if (E <= 32) return launch_gate_mfma_nb<2>(xb, wb, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream);
    return launch_gate_mfma_nb<4>(xb, wb, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream);
}

template <typename T, int EMAX, int NCH, int TPW>
static hipError_t launch_gate_cfg(const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                                  int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                  hipStream_t stream)
{
    const int tokens_per_block = 4 * TPW;
    const int blocks = (T_tok + tokens_per_block - 1) / tokens_per_block;
    const size_t w_bytes = static_cast<size_t>(E) * d * sizeof(T);
    if (w_bytes <= 64 * 1024) {
        hipLaunchKernelGGL((gate_kernel<T, EMAX, NCH, TPW, true>), dim3(blocks), dim3(256), w_bytes, stream,
                           static_cast<const T*>(x), static_cast<const T*>(Wg), bg, T_tok, d, E, k, n_shared, renorm,
                           scores, idx, probs, logits);
    } else {
        hipLaunchKernelGGL((gate_kernel<T, EMAX, NCH, TPW, false>), dim3(blocks), dim3(256), 0, stream,
                           static_cast<const T*>(x), static_cast<const T*>(Wg), bg, T_tok, d, E, k, n_shared, renorm,
                           scores, idx, probs, logits);
    }
    return hipGetLastError();
}

// NCH = 16-byte slices per lane and row (ceil(d / V / 64)); TPW shrinks as the per-lane state grows
template <typename T, int EMAX, int TPW>
static hipError_t launch_gate_e(const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                                int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                hipStream_t stream, bool* ok)
{
    const int nch = (d / Store<T>::kVec + kWave - 1) / kWave;
    *ok = true;
#define DICEMOE_GATE_CASE(N_, TPW_) \
    return launch_gate_cfg<T, EMAX, N_, TPW_>(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream)
    if (nch <= 1) DICEMOE_GATE_CASE(1, TPW);
    if (nch <= 2) DICEMOE_GATE_CASE(2, TPW);
    if (nch <= 3) DICEMOE_GATE_CASE(3, TPW);
    if (nch <= 4) DICEMOE_GATE_CASE(4, TPW);
    if (nch <= 8) DICEMOE_GATE_CASE(8, (TPW > 2 ? 2 : TPW));
    if (nch <= 16) DICEMOE_GATE_CASE(16, 1);
#undef DICEMOE_GATE_CASE
    *ok = false;
    return hipSuccess;
}

template <typename T>
static hipError_t launch_gate_t(const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                                int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                                hipStream_t stream, bool* ok)
{
    if (E <= 8) return launch_gate_e<T, 8, 4>(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream, ok);
    if (E <= 16) return launch_gate_e<T, 16, 2>(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream, ok);
    if (E <= 32) return launch_gate_e<T, 32, 1>(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream, ok);
    return launch_gate_e<T, 64, 1>(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream, ok);
}

hipError_t launch_gate(bool bf16, const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                       int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits, hipStream_t stream)
{
    if (bf16) return launch_gate_mfma(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream);
    bool ok = true;
    hipError_t err = launch_gate_t<float>(x, Wg, bg, T_tok, d, E, k, n_shared, renorm, scores, idx, probs, logits, stream, &ok);
    if (!ok) return hipErrorInvalidValue;     // float rows beyond 16 slices per lane (4096 columns)
    return err;
}

}  // namespace dicemoe
