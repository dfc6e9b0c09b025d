// C-ABI of the library: argument validation on the host, then the kernel launchers.
// See include/dice_moe.h for the meaning of every argument.
#include "../../include/dice_moe.h"

#include <cstdio>
#include <cstring>
#include <new>

#include "kernels.hpp"

struct moe_ctx {
    moe_shape shape;
    char err[256];
    uint64_t ffn_ready;     // bit v: the FFN kernels' per-device attributes have been set on device v
    hipEvent_t ffn_between; // profiling aid: recorded between the two GEMMs of every expert FFN call (or null)
};

namespace {

using namespace dicemoe;

int fail(moe_ctx* ctx, int status, const char* fmt, long a = 0, long b = 0)
{
    if (ctx) std::snprintf(ctx->err, sizeof(ctx->err), fmt, a, b);
    return status;
}

int hip_result(moe_ctx* ctx, hipError_t err, const char* what)
{
    if (err == hipSuccess) return MOE_OK;
    if (ctx) std::snprintf(ctx->err, sizeof(ctx->err), "%s: %s", what, hipGetErrorString(err));
    return MOE_ERR_HIP;
}

bool is_bf16(const moe_ctx* ctx) { return ctx->shape.dtype == MOE_BF16; }
// slots per token and expert ids in use, shared experts included
int slots(const moe_ctx* ctx) { return ctx->shape.k + ctx->shape.n_shared; }
int experts(const moe_ctx* ctx) { return ctx->shape.E + ctx->shape.n_shared; }
size_t elem_bytes(const moe_ctx* ctx) { return is_bf16(ctx) ? 2 : 4; }
// workspace: [hidden activations of the FFN, rows x F][float partial sums of a split second GEMM (bf16 only)]
size_t hidden_bytes(const moe_ctx* ctx)
{
    const size_t rows = static_cast<size_t>(ctx->shape.T_max) * slots(ctx);
    return ((rows * ctx->shape.F * elem_bytes(ctx) + 255) / 256) * 256;
}

// the two status words of the FFN's launch check sit behind the hidden activations and the partial sums
// (the dispatch scratch shares the start of the workspace with the hidden activations: the calls of one
// workspace run in stream order)
size_t status_offset(const moe_ctx* ctx)
{
    size_t front = hidden_bytes(ctx);
    const size_t disp = dicemoe::dispatch_scratch_bytes(static_cast<long long>(ctx->shape.T_max) * slots(ctx), experts(ctx));
    if (disp > front) front = (disp + 255) / 256 * 256;
    return front + (is_bf16(ctx) ? dicemoe::kSplitKBytes : 0);
}

int check_T(moe_ctx* ctx, int32_t T)
{
    if (T < 0 || T > ctx->shape.T_max) return fail(ctx, MOE_ERR_SHAPE, "T=%ld outside 0..T_max=%ld", T, ctx->shape.T_max);
    return MOE_OK;
}

// Validates a refresh policy for T tokens and counts the routed pairs it refreshes (Algorithm 4:
// slot 0 always, the other slots when step_t % stride_n == 0; the fraction forms by definition).
int policy_routed_pairs(moe_ctx* ctx, const moe_policy* policy, int32_t T, int32_t* routed)
{
    const int k = ctx->shape.k;
    const long N = static_cast<long>(T) * k;
    switch (policy->kind) {
    case MOE_REFRESH_ALL: *routed = static_cast<int32_t>(N); return MOE_OK;
    case MOE_REFRESH_NONE: *routed = 0; return MOE_OK;
    case MOE_REFRESH_ALG4:
    case MOE_REFRESH_ALG4_HIGH:
    case MOE_REFRESH_ALG4_RANDOM:
        if (policy->stride_n < 1 || policy->step_t < 0)
            return fail(ctx, MOE_ERR_POLICY, "ALG4 needs step_t >= 0 and stride_n >= 1 (got %ld, %ld)",
                        policy->step_t, policy->stride_n);
        *routed = (policy->step_t % policy->stride_n == 0) ? static_cast<int32_t>(N) : T;
        return MOE_OK;
    case MOE_REFRESH_FRACTION_TOKEN:
        if (policy->n_units < 0 || policy->n_units > T)
            return fail(ctx, MOE_ERR_POLICY, "FRACTION_TOKEN n_units=%ld outside 0..T=%ld", policy->n_units, T);
        *routed = policy->n_units * k;
        return MOE_OK;
    case MOE_REFRESH_FRACTION_PAIR:
        if (policy->n_units < 0 || policy->n_units > N)
            return fail(ctx, MOE_ERR_POLICY, "FRACTION_PAIR n_units=%ld outside 0..T*k=%ld", policy->n_units, N);
        *routed = policy->n_units;
        return MOE_OK;
    default:
        return fail(ctx, MOE_ERR_POLICY, "unknown policy kind %ld", policy->kind);
    }
}

}  // namespace

extern "C" {

int moe_create(moe_ctx** out, const moe_shape* s)
{
    if (!out || !s) return MOE_ERR_NULL;
    *out = nullptr;
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (s->T_max < 0 || s->d < 1 || s->F < 1 || s->E < 1 || s->k < 1) return MOE_ERR_SHAPE;
    if (s->n_shared < 0 || s->k > s->E || s->E + s->n_shared > 64) return MOE_ERR_SHAPE;
    const int mult = (s->dtype == MOE_BF16) ? 64 : 16;
    if (s->d % mult != 0 || s->F % mult != 0) return MOE_ERR_SHAPE;
    if (s->dtype == MOE_F32 && s->d > 4096) return MOE_ERR_SHAPE;     // the float router holds a row in 16 slices per lane
    const long long rows = static_cast<long long>(s->T_max) * (s->k + s->n_shared);
    const long long widest = s->d > s->F ? s->d : s->F;
    if (rows * widest >= (1ll << 31)) return MOE_ERR_SHAPE;
    if (static_cast<long long>(s->T_max) * s->E >= (1ll << 31)) return MOE_ERR_SHAPE;
    moe_ctx* ctx = new (std::nothrow) moe_ctx;
    if (!ctx) return MOE_ERR_NULL;
    ctx->shape = *s;
    ctx->shape.renorm_topk = s->renorm_topk ? 1 : 0;
    ctx->err[0] = '\0';
    ctx->ffn_ready = 0;
    ctx->ffn_between = nullptr;
    *out = ctx;
    return MOE_OK;
}

int moe_destroy(moe_ctx* ctx)
{
    if (!ctx) return MOE_ERR_NULL;
    delete ctx;
    return MOE_OK;
}

size_t moe_workspace_bytes(const moe_ctx* ctx)
{
    if (!ctx) return 0;
    return status_offset(ctx) + 4096;
}

const char* moe_last_error(const moe_ctx* ctx) { return ctx ? ctx->err : "null context"; }

const char* moe_status_string(int status)
{
    switch (status) {
    case MOE_OK: return "MOE_OK";
    case MOE_ERR_NULL: return "MOE_ERR_NULL";
    case MOE_ERR_SHAPE: return "MOE_ERR_SHAPE";
    case MOE_ERR_DTYPE: return "MOE_ERR_DTYPE";
    case MOE_ERR_POLICY: return "MOE_ERR_POLICY";
    case MOE_ERR_WORKSPACE: return "MOE_ERR_WORKSPACE";
    case MOE_ERR_CACHE_COLD: return "MOE_ERR_CACHE_COLD";
    case MOE_ERR_HIP: return "MOE_ERR_HIP";
    default: return "MOE_ERR_UNKNOWN";
    }
}

int moe_gate(moe_ctx* ctx, const void* x, const void* Wg, const float* bg, int32_t T, float* scores,
             int32_t* expert_idx, float* probs_all, float* logits, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!x || !Wg || !scores || !expert_idx) return fail(ctx, MOE_ERR_NULL, "moe_gate: null pointer");
    if (T == 0) return MOE_OK;
    const moe_shape& s = ctx->shape;
    return hip_result(ctx,
                      launch_gate(is_bf16(ctx), x, Wg, bg, T, s.d, s.E, s.k, s.n_shared, s.renorm_topk, scores,
                                  expert_idx, probs_all, logits, static_cast<hipStream_t>(stream)),
                      "moe_gate");
}

int moe_policy_refreshed_pairs(moe_ctx* ctx, const moe_policy* policy, int32_t T, int32_t* n_pairs,
                               int32_t* n_routed)
{
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!policy || !n_pairs) return fail(ctx, MOE_ERR_NULL, "moe_policy_refreshed_pairs: null pointer");
    int32_t routed = 0;
    if (int rc = policy_routed_pairs(ctx, policy, T, &routed)) return rc;
    *n_pairs = routed + T * ctx->shape.n_shared;
    if (n_routed) *n_routed = routed;
    return MOE_OK;
}

int moe_conditional_refresh(moe_ctx* ctx, const float* scores, const int32_t* expert_idx, int32_t T,
                            const moe_policy* policy, uint8_t* mask, int32_t* n_refresh, void* workspace,
                            void* stream)
{
    (void)expert_idx;      // no current policy reads the expert ids or needs scratch (see the header)
    (void)workspace;
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!policy || !mask || !n_refresh) return fail(ctx, MOE_ERR_NULL, "moe_conditional_refresh: null pointer");
    int32_t routed = 0;
    if (int rc = policy_routed_pairs(ctx, policy, T, &routed)) return rc;
    const moe_shape& s = ctx->shape;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n_value = routed + T * s.n_shared;       // what the device-side n_refresh receives
    const long N = static_cast<long>(T) * s.k;
    switch (policy->kind) {
    case MOE_REFRESH_ALL:
    case MOE_REFRESH_NONE:
        return hip_result(ctx, launch_refresh_simple(policy->kind, T, s.k, s.n_shared, 0, 0u, n_value, mask, n_refresh, st),
                          "moe_conditional_refresh");
    case MOE_REFRESH_ALG4:
    case MOE_REFRESH_ALG4_HIGH:
    case MOE_REFRESH_ALG4_RANDOM:
        return hip_result(ctx,
                          launch_refresh_simple(policy->kind, T, s.k, s.n_shared,
                                                policy->step_t % policy->stride_n != 0 ? 1 : 0,
                                                static_cast<uint32_t>(policy->n_units), n_value, mask, n_refresh, st),
                          "moe_conditional_refresh");
    case MOE_REFRESH_FRACTION_TOKEN:
        if (!scores) return fail(ctx, MOE_ERR_NULL, "moe_conditional_refresh: scores is null");
        return hip_result(ctx,
                          launch_refresh_select(scores, T, s.k, s.n_shared, 0, policy->n_units, true, n_value, mask,
                                                n_refresh, st),
                          "moe_conditional_refresh");
    default: {      // MOE_REFRESH_FRACTION_PAIR (policy_routed_pairs has rejected every other kind)
        if (!scores) return fail(ctx, MOE_ERR_NULL, "moe_conditional_refresh: scores is null");
        if (policy->n_units == N)
            return hip_result(ctx, launch_refresh_simple(MOE_REFRESH_ALL, T, s.k, s.n_shared, 0, 0u, n_value, mask, n_refresh, st),
                              "moe_conditional_refresh");
        // slots before `slot` are refreshed for every token, slot `slot` for its m best tokens
        const int slot = T > 0 ? policy->n_units / T : 0;
        const int m = T > 0 ? policy->n_units % T : 0;
        return hip_result(ctx,
                          launch_refresh_select(scores, T, s.k, s.n_shared, slot, m, false, n_value, mask, n_refresh, st),
                          "moe_conditional_refresh");
    }
    }
}

int moe_dispatch(moe_ctx* ctx, const void* x, const int32_t* expert_idx, const uint8_t* mask, int32_t T,
                 void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv, void* workspace,
                 void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!expert_idx || !counts || !offsets || !perm || !inv || (x_packed && !x))
        return fail(ctx, MOE_ERR_NULL, "moe_dispatch: null pointer");
    const moe_shape& s = ctx->shape;
    // the per-workgroup counts travel from the counting launch to the placing launch at the start of the workspace
    if (!workspace && dicemoe::dispatch_scratch_bytes(static_cast<long long>(T) * slots(ctx), experts(ctx)) > 0)
        return fail(ctx, MOE_ERR_WORKSPACE, "moe_dispatch: workspace is null");
    return hip_result(ctx,
                      launch_dispatch(is_bf16(ctx), x, expert_idx, mask, T, s.d, experts(ctx), slots(ctx), x_packed, counts, offsets,
                                      perm, inv, static_cast<int32_t*>(workspace), static_cast<hipStream_t>(stream)),
                      "moe_dispatch");
}

int moe_dispatch_noalloc(moe_ctx* ctx, const void* x, const int32_t* expert_idx, const uint8_t* mask, int32_t T,
                         void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!expert_idx || !counts || !offsets || !perm || !inv || (x_packed && !x))
        return fail(ctx, MOE_ERR_NULL, "moe_dispatch_noalloc: null pointer");
    const moe_shape& s = ctx->shape;
    const size_t need = dicemoe::dispatch_scratch_bytes(static_cast<long long>(T) * slots(ctx), experts(ctx));
    if (need > dicemoe::dispatch_static_scratch_bytes())
        return fail(ctx, MOE_ERR_SHAPE, "moe_dispatch_noalloc: this T needs %ld bytes of scratch, the library's static buffer holds %ld",
                    static_cast<long>(need), static_cast<long>(dicemoe::dispatch_static_scratch_bytes()));
    int32_t* scratch_ptr = nullptr;
    if (hipError_t err = dicemoe::dispatch_static_scratch(&scratch_ptr); err != hipSuccess)
        return hip_result(ctx, err, "moe_dispatch_noalloc");
    return hip_result(ctx,
                      launch_dispatch(is_bf16(ctx), x, expert_idx, mask, T, s.d, experts(ctx), slots(ctx), x_packed, counts, offsets,
                                      perm, inv, scratch_ptr, static_cast<hipStream_t>(stream)),
                      "moe_dispatch_noalloc");
}

}  // extern "C"

static int expert_ffn_common(moe_ctx* ctx, const char* who, const void* x_rows, const int32_t* row_pairs,
                             const int32_t* seg_offsets, const int32_t* seg_expert, int32_t n_segments,
                             int32_t max_rows, const void* W1, const float* b1, const void* W2, const float* b2,
                             void* h_packed, const int32_t* out_pairs, void* workspace, void* stream)
{
    const moe_shape& s = ctx->shape;
    if (n_segments < 1 || n_segments > 1024)
        return fail(ctx, MOE_ERR_SHAPE, "n_segments=%ld outside 1..1024", n_segments);
    if (max_rows < 0 || static_cast<long long>(max_rows) > static_cast<long long>(s.T_max) * slots(ctx))
        return fail(ctx, MOE_ERR_SHAPE, "max_rows=%ld outside 0..T_max*slots=%ld", max_rows, static_cast<long>(s.T_max) * slots(ctx));
    if (!x_rows || !seg_offsets || !seg_expert || !W1 || !W2 || !h_packed) {
        std::snprintf(ctx->err, sizeof(ctx->err), "%s: null pointer", who);
        return MOE_ERR_NULL;
    }
    if (!workspace) {
        std::snprintf(ctx->err, sizeof(ctx->err), "%s: workspace is null", who);
        return MOE_ERR_WORKSPACE;
    }
    // per-device kernel attributes, once per context and device (a context serves one host thread at a time)
    int device = 0;
    if (hipError_t err = hipGetDevice(&device); err != hipSuccess) return hip_result(ctx, err, who);
    const bool tracked = device >= 0 && device < 64;
    if (!tracked || !((ctx->ffn_ready >> device) & 1u)) {
        if (hipError_t err = dicemoe::prepare_expert_ffn(); err != hipSuccess) return hip_result(ctx, err, who);
        if (tracked) ctx->ffn_ready |= 1ull << device;
    }
    char* ws = static_cast<char*>(workspace);
    return hip_result(ctx,
                      launch_expert_ffn(is_bf16(ctx), x_rows, row_pairs, slots(ctx), seg_offsets, seg_expert, n_segments,
                                        max_rows, s.d, s.F, W1, b1, W2, b2, h_packed, out_pairs, workspace,
                                        is_bf16(ctx) ? ws + status_offset(ctx) - dicemoe::kSplitKBytes : nullptr,
                                        is_bf16(ctx) ? dicemoe::kSplitKBytes : 0,
                                        reinterpret_cast<int32_t*>(ws + status_offset(ctx)), static_cast<hipStream_t>(stream),
                                        ctx->ffn_between),
                      who);
}

extern "C" {

int moe_expert_ffn(moe_ctx* ctx, const void* x_packed, const int32_t* seg_offsets, const int32_t* seg_expert,
                   int32_t n_segments, int32_t max_rows, const void* W1, const float* b1, const void* W2,
                   const float* b2, void* h_packed, void* workspace, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    return expert_ffn_common(ctx, "moe_expert_ffn", x_packed, nullptr, seg_offsets, seg_expert, n_segments, max_rows, W1,
                             b1, W2, b2, h_packed, nullptr, workspace, stream);
}

int moe_expert_ffn_rows(moe_ctx* ctx, const void* x, const int32_t* row_pairs, const int32_t* seg_offsets,
                        const int32_t* seg_expert, int32_t n_segments, int32_t max_rows, const void* W1,
                        const float* b1, const void* W2, const float* b2, void* h_packed, void* workspace,
                        void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (!row_pairs) return fail(ctx, MOE_ERR_NULL, "moe_expert_ffn_rows: row_pairs is null");
    return expert_ffn_common(ctx, "moe_expert_ffn_rows", x, row_pairs, seg_offsets, seg_expert, n_segments, max_rows, W1,
                             b1, W2, b2, h_packed, nullptr, workspace, stream);
}

int moe_expert_ffn_commit(moe_ctx* ctx, const void* x_rows, const int32_t* row_pairs, const int32_t* out_pairs,
                          const int32_t* seg_offsets, const int32_t* seg_expert, int32_t n_segments, int32_t max_rows,
                          const void* W1, const float* b1, const void* W2, const float* b2, const float* scores,
                          const uint8_t* mask, int32_t T, void* H_buffer, float* S_buffer, void* workspace,
                          void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!out_pairs || !H_buffer || ((scores == nullptr) != (S_buffer == nullptr)))
        return fail(ctx, MOE_ERR_NULL, "moe_expert_ffn_commit: null pointer");
    if (int rc = expert_ffn_common(ctx, "moe_expert_ffn_commit", x_rows, row_pairs, seg_offsets, seg_expert, n_segments,
                                   max_rows, W1, b1, W2, b2, H_buffer, out_pairs, workspace, stream))
        return rc;
    if (!scores) return MOE_OK;              // the scores stay with the caller (moe_combine writes them through)
    return hip_result(ctx,
                      launch_commit_scores(scores, mask, T, slots(ctx), ctx->shape.k, S_buffer,
                                           static_cast<hipStream_t>(stream)),
                      "moe_expert_ffn_commit");
}

int moe_expert_ffn_between_event(moe_ctx* ctx, void* event)
{
    if (!ctx) return MOE_ERR_NULL;
    ctx->ffn_between = static_cast<hipEvent_t>(event);
    return MOE_OK;
}

int moe_calibrate_copy(void* dst, const void* src, size_t bytes, int32_t workgroups, void* stream)
{
    if (!dst || !src) return MOE_ERR_NULL;
    if (bytes % 16 != 0 || workgroups < 1) return MOE_ERR_SHAPE;
    return dicemoe::launch_calibrate_copy(dst, src, bytes, workgroups, static_cast<hipStream_t>(stream)) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_calibrate_mfma(const void* operands, float* sink, int32_t iters, int32_t workgroups, void* stream)
{
    if (!operands || !sink) return MOE_ERR_NULL;
    if (iters < 1 || workgroups < 1) return MOE_ERR_SHAPE;
    return dicemoe::launch_calibrate_mfma(operands, sink, iters, workgroups, static_cast<hipStream_t>(stream)) == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_expert_ffn_status(moe_ctx* ctx, const void* workspace, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (!workspace) return fail(ctx, MOE_ERR_WORKSPACE, "moe_expert_ffn_status: workspace is null");
    int32_t words[2] = {0, 0};
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t err = hipMemcpyAsync(words, static_cast<const char*>(workspace) + status_offset(ctx), sizeof(words),
                                    hipMemcpyDeviceToHost, st);
    if (err == hipSuccess) err = hipStreamSynchronize(st);
    if (err != hipSuccess) return hip_result(ctx, err, "moe_expert_ffn_status");
    if (words[0] != 0)
        return fail(ctx, MOE_ERR_SHAPE, "expert FFN: the segment table held %ld rows but max_rows was %ld; rows beyond it were not computed",
                    words[0], words[1]);
    return MOE_OK;
}

int moe_combine(moe_ctx* ctx, const void* h_packed, const int32_t* inv, const float* scores, const uint8_t* mask,
                int32_t T, void* H_cache, float* S_cache, int32_t use_fresh_scores, void* y, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (int rc = check_T(ctx, T)) return rc;
    if (!inv || !scores || !y) return fail(ctx, MOE_ERR_NULL, "moe_combine: null pointer");
    if (!h_packed && (!H_cache || ctx->shape.n_shared != 0))
        return fail(ctx, MOE_ERR_NULL, "moe_combine: h_packed may be null only with a cache and without shared experts");
    if (mask && (!H_cache || !S_cache))
        return fail(ctx, MOE_ERR_CACHE_COLD, "moe_combine: a refresh mask was given without a cache");
    if ((H_cache == nullptr) != (S_cache == nullptr))
        return fail(ctx, MOE_ERR_NULL, "moe_combine: H_cache and S_cache must be given together");
    const moe_shape& s = ctx->shape;
    return hip_result(ctx,
                      launch_combine(is_bf16(ctx), h_packed, inv, scores, mask, T, s.d, slots(ctx), s.k, H_cache,
                                     S_cache,
                                     use_fresh_scores ? 1 : 0, y, static_cast<hipStream_t>(stream)),
                      "moe_combine");
}

int moe_ep_segments(moe_ctx* ctx, const int32_t* recv_counts, int32_t W, int32_t E_loc, int32_t* seg_offsets,
                    int32_t* seg_expert, void* stream)
{
    if (!ctx) return MOE_ERR_NULL;
    if (W < 1 || E_loc < 1 || static_cast<long long>(W) * E_loc > 1024 || E_loc > ctx->shape.E)
        return fail(ctx, MOE_ERR_SHAPE, "moe_ep_segments: W=%ld, E_loc=%ld out of range", W, E_loc);
    if (!recv_counts || !seg_offsets || !seg_expert) return fail(ctx, MOE_ERR_NULL, "moe_ep_segments: null pointer");
    return hip_result(ctx,
                      launch_ep_segments(recv_counts, W * E_loc, E_loc, seg_offsets, seg_expert,
                                         static_cast<hipStream_t>(stream)),
                      "moe_ep_segments");
}

}  // extern "C"
