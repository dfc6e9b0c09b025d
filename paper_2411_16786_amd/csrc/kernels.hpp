// Host-side launchers of the gfx950 kernels (one per translation unit); the C-ABI in api.hip
// validates arguments and calls these.  Every launcher only enqueues work on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dicemoe {

// scores / idx have k + n_shared columns: the k routed slots, then slot k+s = (expert E+s, score 1)
hipError_t launch_gate(bool bf16, const void* x, const void* Wg, const float* bg, int T_tok, int d, int E, int k,
                       int n_shared, int renorm, float* scores, int32_t* idx, float* probs, float* logits,
                       hipStream_t stream);

// kind: 0 all, 1 / 5 / 6 Algorithm 4 and its ablation variants, 4 none (elementwise policies); off_step:
// step_t % stride_n != 0.  mask has k + n_shared columns; the shared slots are refreshed under every
// policy.  n_value is written to n_refresh (the refreshed pairs, shared slots included).
hipError_t launch_refresh_simple(int kind, int T_tok, int k, int n_shared, int off_step, uint32_t seed, int n_value,
                                 uint8_t* mask, int32_t* n_refresh, hipStream_t stream);
// exact top-m selection of tokens by scores[i*k + slot] (descending, ties to the lower token);
// token_mode: selected tokens get all k slots; otherwise slots < slot are all refreshed, slot
// `slot` follows the selection and later slots are not refreshed
hipError_t launch_refresh_select(const float* scores, int T_tok, int k, int n_shared, int slot, int m,
                                 bool token_mode, int n_value, uint8_t* mask, int32_t* n_refresh,
                                 hipStream_t stream);

// scratch: dispatch_scratch_bytes(T_tok * k, E) bytes of device memory (per-workgroup expert counts handed
// from the counting launch to the placing launch); may be null when that size is 0
hipError_t launch_dispatch(bool bf16, const void* x, const int32_t* idx, const uint8_t* mask, int T_tok, int d,
                           int E, int k, void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm,
                           int32_t* inv, int32_t* scratch, hipStream_t stream);
size_t dispatch_scratch_bytes(long long n_pairs, int E);
// The library's own scratch for launch_dispatch: a file-scope device array of dispatch_static_scratch_bytes()
// bytes; *out receives its address on the current device (looked up once per device).  No allocation.
size_t dispatch_static_scratch_bytes();
hipError_t dispatch_static_scratch(int32_t** out);

hipError_t launch_combine(bool bf16, const void* h_packed, const int32_t* inv, const float* scores,
                          const uint8_t* mask, int T_tok, int d, int k, int k_cached, void* H_cache,
                          float* S_cache, int use_fresh, void* y, hipStream_t stream);

// x_rows is the packed buffer (row_index == nullptr) or the token matrix with row_index[r] / row_div
// naming the row that packed row r reads; the h row of packed row r is written to row r of h_out, or
// to row out_index[r] when out_index is given (scatter into a buffer indexed by pair id)
hipError_t launch_expert_ffn(bool bf16, const void* x_rows, const int32_t* row_index, int row_div,
                             const int32_t* seg_offsets, const int32_t* seg_expert, int n_seg, int max_rows, int d,
                             int F, const void* W1, const float* b1, const void* W2, const float* b2, void* h_out,
                             const int32_t* out_index, void* hidden, void* partial, size_t partial_bytes,
                             int32_t* status, hipStream_t stream, hipEvent_t between = nullptr);
// between: if given, recorded on the stream after the first GEMM has been enqueued (per-GEMM timing)
// status (two int32 on the device, may be null): written by the first GEMM of every call, see
// report_row_overflow in ffn_mfma.hpp.
// Once per device before the first launch_expert_ffn there: raises the dynamic-LDS limit of the wide kernels.
hipError_t prepare_expert_ffn();

// bytes of float partial sums that the split reduction of the second GEMM may use (beyond `hidden`)
// (at most about 270 workgroups of 128 x 192 float tiles)
constexpr size_t kSplitKBytes = static_cast<size_t>(288) * 128 * 192 * sizeof(float);

// S_buffer[p] = scores[p] for the routed slots (j < k_cached) of every pair with mask[p] != 0 (all if mask is null)
hipError_t launch_commit_scores(const float* scores, const uint8_t* mask, int T_tok, int k, int k_cached,
                                float* S_buffer, hipStream_t stream);

// measurement aids (calibrate.hip): a plain copy of `bytes` (multiple of 16) and a register-resident MFMA loop
// (operands: 16 x 256 x 96 bytes of bf16 bit patterns; flops = workgroups * 4 * iters * 8 * 32768)
hipError_t launch_calibrate_copy(void* dst, const void* src, size_t bytes, int workgroups, hipStream_t stream);
hipError_t launch_calibrate_mfma(const void* operands, float* sink, int iters, int workgroups, hipStream_t stream);

hipError_t launch_ep_segments(const int32_t* recv_counts, int n_seg, int E_loc, int32_t* seg_offsets,
                              int32_t* seg_expert, hipStream_t stream);

}  // namespace dicemoe
