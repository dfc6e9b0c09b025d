/*
 * dice_moe.h -- C-ABI of the MI355X (gfx950) MoE expert layer with DICE's token-level
 * Conditional Communication.
 *
 * The calls follow the paper's statement of one MoE layer under expert parallelism
 * (supplement, Algorithm 1):
 *     [s, idx] <- router(x)            moe_gate
 *     x_d <- all2all_dispatch(x, idx)  moe_dispatch      (one device: group rows by expert)
 *     x_e <- expert(x_d)               moe_expert_ffn
 *     x_c <- all2all_combine(x_e)      moe_combine       (one device: back to token order)
 *     x   <- scale(x_c, s)             moe_combine       (y_i = sum_e s_i^e h_i^e, Section 4.3)
 * and the per-pair transmit/reuse decision of Conditional Communication (supplement,
 * Algorithm 4) sits between router and dispatch:      moe_conditional_refresh.
 * moe_expert_ffn_rows is moe_expert_ffn with the dispatch gather folded in; moe_expert_ffn_commit
 * is the expert call of the asynchronous schedules (supplement, Algorithms 2 and 3), whose results
 * go into the persistent combine buffer for the next step; moe_ep_segments describes an
 * expert-parallel receive buffer to moe_expert_ffn.
 *
 * Conventions for every entry point
 *   - Returns MOE_OK (0) or a negative moe_status.  Never throws, aborts, allocates device
 *     memory or synchronises the host (moe_expert_ffn_status excepted: it waits for the stream).
 *     A context is used by one host thread at a time.  All work is enqueued on `stream` (a hipStream_t passed
 *     as void*; NULL = the default stream) of the current device.
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned, row-major
 *     and contiguous.  moe_shape / moe_policy pointers are HOST pointers read during the call.
 *   - Errors that the host can see (null pointer, bad shape, bad policy, cold cache) return
 *     before anything is launched; a failed launch returns MOE_ERR_HIP.  The text of the last
 *     error of a context is available from moe_last_error().
 *   - Data-dependent sizes (per-expert counts, number of refreshed pairs) stay on the device;
 *     buffers are sized for the worst case N = T*k rows.
 *   - Notation: T tokens, d hidden size, F expert width, E experts, k experts per token,
 *     pair p = i*k + j = (token i, slot j); slot 0 is the token's top-1 expert.
 *   - Storage type `dtype` applies to x, Wg, W1, W2, x_packed, h_packed, H_cache and y.
 *     Scores, probabilities, logits and biases are always float; indices are int32.
 *   - Weights are stored like a linear layer's weight, rows = output features:
 *       Wg[E][d],  W1[E][F][d],  b1[E][F],  W2[E][d][F],  b2[E][d].
 *   - Limits: 1 <= k <= E, E + n_shared <= 64; d % 16 == 0 and F % 16 == 0; for MOE_BF16 also d % 64 == 0 and
 *     F % 64 == 0 (MFMA tile depth); for MOE_F32 d <= 4096; T*k < 2^31 / max(d, F).
 */
#ifndef DICE_MOE_H
#define DICE_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_NULL = -1,       /* a required pointer is NULL */
    MOE_ERR_SHAPE = -2,      /* a size is out of range or violates a limit above */
    MOE_ERR_DTYPE = -3,      /* unknown storage type */
    MOE_ERR_POLICY = -4,     /* refresh policy fields out of range */
    MOE_ERR_WORKSPACE = -5,  /* workspace pointer missing */
    MOE_ERR_CACHE_COLD = -6, /* a partial refresh was asked for but no cache was given */
    MOE_ERR_HIP = -7         /* the HIP runtime refused a launch */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;

typedef struct {
    int32_t T_max;       /* largest token count of any call; packed buffers hold T_max*k rows */
    int32_t d, F, E, k;
    int32_t dtype;       /* moe_dtype */
    int32_t renorm_topk; /* 0: scores are the softmax over all E experts taken at the selected
                            ones (default; the paper only says "router scores");
                            1: additionally divided by their sum over the k selected */
    int32_t n_shared;    /* shared experts of the DiT-MoE layer (model description: experts that every
                            token uses, always fresh, unscaled).  They are carried as n_shared extra
                            slots per token behind the k routed ones: slot k+s of every token goes to
                            expert id E+s with score 1 and is refreshed under every policy.  All
                            per-pair arrays then have k + n_shared columns and the expert weights
                            hold E + n_shared experts (shared ones last); E + n_shared <= 64.
                            0 = routed experts only. */
} moe_shape;

/* Which (token, slot) pairs are recomputed ("transmitted") in this step; the others reuse the
 * cached expert output of an earlier step (Algorithm 4). */
typedef enum {
    MOE_REFRESH_ALL = 0,            /* synchronous layer: every pair */
    MOE_REFRESH_ALG4 = 1,           /* Algorithm 4: slot 0 always; other slots iff step_t % stride_n == 0 */
    MOE_REFRESH_FRACTION_TOKEN = 2, /* the n_units tokens with the largest top-1 score, all their slots */
    MOE_REFRESH_FRACTION_PAIR = 3,  /* the first n_units pairs in the order (slot asc, score desc, token asc) */
    MOE_REFRESH_NONE = 4,           /* no pair: the output is rebuilt from the cache */
    /* Ablation of which pair is deprioritised (Section 5.3, "Conditional Communication"; ablation
     * table rows "High Score" and "Random"): Algorithm 4 with another always-fresh slot. */
    MOE_REFRESH_ALG4_HIGH = 5,      /* slot k-1 (lowest activated score) always; others iff step_t % stride_n == 0 */
    MOE_REFRESH_ALG4_RANDOM = 6     /* one slot per token always, slot = mix32(seed = n_units, token) mod k, where
                                       mix32(s, i): h = s*0x9E3779B9 + i; h ^= h>>16; h *= 0x85EBCA6B; h ^= h>>13;
                                       h *= 0xC2B2AE35; h ^= h>>16 (mod 2^32); others iff step_t % stride_n == 0 */
} moe_policy_kind;

typedef struct {
    int32_t kind;             /* moe_policy_kind */
    int32_t step_t, stride_n; /* ALG4: step_t >= 0, stride_n >= 1 */
    int32_t n_units;          /* FRACTION_TOKEN: 0..T tokens; FRACTION_PAIR: 0..T*k pairs.  The
                                 caller rounds a fraction to this integer.  ALG4_RANDOM: the seed. */
    int32_t use_fresh_scores; /* which score scales a reused cached output (supplement, "Expert
                                 Score Scaling"): 0 = the cached score that belonged to the stale
                                 input (the paper's choice), 1 = this step's score */
} moe_policy;

typedef struct moe_ctx moe_ctx; /* opaque; host memory only (shape, last error) */

/* Create / destroy a context.  `shape` is validated here (MOE_ERR_SHAPE / MOE_ERR_DTYPE). */
int moe_create(moe_ctx** out, const moe_shape* shape);
int moe_destroy(moe_ctx* ctx);

/* Bytes of device workspace that moe_conditional_refresh, moe_dispatch and moe_expert_ffn may
 * use for T_max tokens: the FFN's hidden activations [T_max*k, F], (MOE_BF16) 28 MB of float
 * partial sums for the second GEMM when its reduction is split over several workgroups (few
 * rows), and the status words of moe_expert_ffn_status.  One workspace can serve all three calls of a layer, and all layers, on one stream. */
size_t moe_workspace_bytes(const moe_ctx* ctx);

/* Text of the last error recorded on this context ("" if none); valid until the next call. */
const char* moe_last_error(const moe_ctx* ctx);
/* Name of a status code. */
const char* moe_status_string(int status);

/* In every array below, "k" as a column count (scores, expert_idx, mask, inv, perm, the caches,
 * max_rows' bound T*k) stands for k + n_shared when the shape has shared experts, pair id
 * p = i*(k + n_shared) + j, and W1/b1/W2/b2 hold E + n_shared experts; counts and offsets then
 * have E + n_shared (+1) entries.  moe_gate writes the shared slots (expert E+s, score 1),
 * moe_conditional_refresh sets their mask bytes to 1 and counts them in n_refresh; a mask that
 * clears a shared slot is an error of the caller (moe_combine keeps no cache for those slots
 * and leaves H_cache / S_cache at those positions untouched). */

/* Router (Algorithm 1, "[s, idx] <- router(x)"; K activated experts per token, Conditional
 * Communication figure).  logits z = x . Wg^T (+ bg), accumulated in float; expert_idx[i][j] is
 * the expert with the j-th largest logit of token i, equal logits going to the lower expert id;
 * scores[i][j] = softmax_over_E(z_i)[expert_idx[i][j]] (renormalised over the k if the shape
 * says so).
 *   in : x[T][d], Wg[E][d] (dtype), bg[E] float or NULL
 *   out: scores[T][k] float, expert_idx[T][k] int32,
 *        probs_all[T][E] float or NULL, logits[T][E] float or NULL
 * T may be 0 (nothing is launched). */
int moe_gate(moe_ctx* ctx, const void* x, const void* Wg, const float* bg, int32_t T,
             float* scores, int32_t* expert_idx, float* probs_all, float* logits, void* stream);

/* Conditional Communication decision (Algorithm 4 and its fraction forms, see moe_policy_kind).
 * Ordering is exact on the float bit patterns of `scores`; equal scores go to the lower token.
 *   in : scores[T][k] (read by the FRACTION policies only; the others accept NULL);
 *        expert_idx[T][k]: no current policy reads it, NULL is accepted
 *   out: mask[T][k] uint8 (1 = refresh), n_refresh[1] int32 on the device
 * workspace: no current policy uses it, NULL is accepted (the argument keeps the call's shape
 * stable for policies that need scratch). */
int moe_conditional_refresh(moe_ctx* ctx, const float* scores, const int32_t* expert_idx,
                            int32_t T, const moe_policy* policy, uint8_t* mask,
                            int32_t* n_refresh, void* workspace, void* stream);

/* Number of pairs that `policy` refreshes among T tokens, known on the host without reading the
 * mask back (Algorithm 4: slot 0 of every token always, the other slots on steps with
 * step_t % stride_n == 0; the fraction forms refresh exactly n_units tokens or pairs; shared-expert
 * slots are refreshed for every token in every step).  It is the value moe_conditional_refresh
 * writes to n_refresh, and the bound max_rows that sizes the expert FFN launch of that step.
 *   in : policy (host), T
 *   out: n_pairs (host): refreshed pairs, shared-expert slots included; n_routed (host, may be
 *        NULL): the routed ones among them (n_pairs - T * n_shared)
 * Nothing is launched.  MOE_ERR_POLICY for fields out of range, as in moe_conditional_refresh. */
int moe_policy_refreshed_pairs(moe_ctx* ctx, const moe_policy* policy, int32_t T, int32_t* n_pairs,
                               int32_t* n_routed);

/* Dispatch on one device (Algorithm 1, dispatch): a stable counting sort of the refreshed pairs
 * by expert id and a row gather into an expert-contiguous buffer.  With experts partitioned in
 * blocks over expert-parallel ranks the same order is (destination rank, local expert, token),
 * i.e. `counts` viewed as [W][E/W] are the all-to-all send counts and x_packed is the send buffer.
 *   in : x[T][d], expert_idx[T][k], mask[T][k] or NULL (= every pair)
 *   out: x_packed[R][d] rows of the refreshed pairs ordered by (expert asc, pair id asc), copied
 *        bit for bit (rows >= R are left untouched); counts[E]; offsets[E+1] exclusive prefix
 *        sums (offsets[E] = R); perm[T*k]: pair id of packed row r, -1 for r >= R;
 *        inv[T*k]: packed row of pair p, -1 if p is not refreshed.
 * x_packed may be NULL: then only the index outputs are written (x is not read and may be NULL too)
 * and the rows are gathered by the consumer, see moe_expert_ffn_rows.
 * workspace: moe_workspace_bytes(); at most the first 4 * (E + n_shared) * (ceil(T*k / 256) + 1) bytes carry
 * per-workgroup expert counts between the two launches of the sort (they overlap the expert FFN's
 * hidden activations: calls that share a workspace must run in stream order).  NULL is accepted
 * when T*k <= 2048 (one workgroup sorts alone). */
int moe_dispatch(moe_ctx* ctx, const void* x, const int32_t* expert_idx, const uint8_t* mask,
                 int32_t T, void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm,
                 int32_t* inv, void* workspace, void* stream);

/* moe_dispatch for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The per-workgroup counts that moe_dispatch
 * keeps in the caller's workspace live here in a 64 KiB array inside the library's device code (one
 * per GPU, held until the process ends); the call allocates nothing and returns the same outputs,
 * bit for bit.  Limit: 4 * (E + n_shared) * (workgroups + 1) <= 65536 bytes, where the sort runs on at
 * most 256 workgroups up to 2^19 pairs and on ceil(T*k / 2048) beyond (e.g. E = 8: up to 4 million
 * pairs); beyond it the call returns MOE_ERR_SHAPE and launches nothing.  Every call on a GPU shares
 * that GPU's array: calls that overlap on one GPU (two streams, two threads) race; calls in stream
 * order are safe, and nothing in the array has to be cleared between them (the counting launch writes
 * every entry the placing launch reads). */
int moe_dispatch_noalloc(moe_ctx* ctx, const void* x, const int32_t* expert_idx, const uint8_t* mask,
                         int32_t T, void* x_packed, int32_t* counts, int32_t* offsets, int32_t* perm,
                         int32_t* inv, void* stream);

/* Grouped expert FFN (Algorithm 1, "x_e <- expert(x_d)"; experts are feed-forward networks):
 * for every segment g, rows seg_offsets[g] .. seg_offsets[g+1]-1 of x_packed go through expert
 * seg_expert[g]:  h = W2_e . gelu(W1_e . x + b1_e) + b2_e,  gelu(u) = u/2 (1 + erf(u/sqrt 2)).
 * MOE_BF16: bf16 MFMA with float accumulation, the hidden activation is rounded to bf16 once.
 * Segments generalise the per-expert grouping of moe_dispatch (n_segments = E, seg_offsets =
 * offsets, seg_expert = 0..E-1) to an expert-parallel receive buffer ordered
 * [source rank][local expert] (n_segments = W * E_loc, see moe_ep_segments).
 *   in : x_packed[>= seg_offsets[n_segments]][d]; seg_offsets[n_segments+1], seg_expert[n_segments]
 *        (device); max_rows >= seg_offsets[n_segments] (host bound that sizes the launch,
 *        max_rows <= T_max*k); W1, W2 (dtype); b1, b2 float or NULL; every seg_expert < E
 *   out: h_packed[..][d] (dtype); rows outside every segment are left untouched
 * workspace: moe_workspace_bytes(). 1 <= n_segments <= 1024. */
int moe_expert_ffn(moe_ctx* ctx, const void* x_packed, const int32_t* seg_offsets,
                   const int32_t* seg_expert, int32_t n_segments, int32_t max_rows,
                   const void* W1, const float* b1, const void* W2, const float* b2,
                   void* h_packed, void* workspace, void* stream);

/* The same expert FFN with the dispatch gather folded into its first operand load (single-device
 * path of Algorithm 1: dispatch and expert on one device need no send buffer): packed row r is read
 * from x[row_pairs[r] / k], where row_pairs is the perm output of moe_dispatch (pair id of packed
 * row r), so x_packed is never materialised.  Results are bit-identical to moe_dispatch with a packed
 * buffer followed by moe_expert_ffn.
 *   in : x[T][d] (dtype); row_pairs[>= seg_offsets[n_segments]] (device), every entry in 0..T*k-1;
 *        the other arguments as for moe_expert_ffn */
int moe_expert_ffn_rows(moe_ctx* ctx, const void* x, const int32_t* row_pairs,
                        const int32_t* seg_offsets, const int32_t* seg_expert, int32_t n_segments,
                        int32_t max_rows, const void* W1, const float* b1, const void* W2,
                        const float* b2, void* h_packed, void* workspace, void* stream);

/* Expert FFN whose results go straight into the persistent combine buffer, for the asynchronous
 * schedules (Algorithm 3, "async_combine" of the expert outputs, waited for in the next step;
 * Algorithm 2 likewise; Section 4.1: only the combined results are buffered for the next step).
 * The h row of packed row r is written to H_buffer[out_pairs[r]] (a row per pair id, the layout of
 * moe_combine's H_cache) instead of a packed buffer, and S_buffer[p] = scores[p] for the routed
 * slots of every pair with mask[p] != 0 (all of them if mask is NULL): after the call the buffers
 * hold this step's results for the refreshed pairs and the older ones for the rest, which is what
 * moe_combine reads in the next step when it is given a mask that refreshes nothing.
 *   in : x_rows: the packed rows (row_pairs NULL) or x[T][d] read through row_pairs as in
 *        moe_expert_ffn_rows; out_pairs[>= seg_offsets[n_segments]] (device), the pair id of
 *        each packed row (moe_dispatch's perm), every entry in 0..T_max*k-1 and distinct;
 *        scores[T][k], mask[T][k] or NULL: those of the step the packed rows were dispatched in;
 *        the other arguments as for moe_expert_ffn
 *   io : H_buffer[T_max*k][d] (dtype), S_buffer[T_max*k] float; rows and scores of pairs that
 *        are not named stay as they are
 * The caller orders this call after the moe_combine that still reads the old buffer contents.
 * scores and S_buffer may both be NULL: then only the rows are written (the synchronous layer with a
 * cache uses this: its moe_combine, called afterwards with h_packed = NULL, reads every row from the
 * cache and writes the scores through itself, so refreshed rows cross memory once instead of twice). */
int moe_expert_ffn_commit(moe_ctx* ctx, const void* x_rows, const int32_t* row_pairs,
                          const int32_t* out_pairs, const int32_t* seg_offsets,
                          const int32_t* seg_expert, int32_t n_segments, int32_t max_rows,
                          const void* W1, const float* b1, const void* W2, const float* b2,
                          const float* scores, const uint8_t* mask, int32_t T, void* H_buffer,
                          float* S_buffer, void* workspace, void* stream);

/* Launch check of the expert FFN calls.  Segment sizes live on the device, so the three calls above
 * size their launch from the host bound max_rows; if the segment table holds more rows than that,
 * the rows beyond the launched tiles are NOT computed.  Every FFN call records the comparison in
 * its workspace; this call waits for `stream` (it is the one entry point that synchronises the
 * host) and reports what the LAST expert FFN call enqueued with this workspace found:
 * MOE_OK, or MOE_ERR_SHAPE with the two numbers in moe_last_error().  The workspace must have been
 * used by at least one expert FFN call of this context's shape. */
int moe_expert_ffn_status(moe_ctx* ctx, const void* workspace, void* stream);

/* Measurement aids (they compute nothing of the method; the benchmark uses them to print the
 * per-GEMM split of the expert FFN and the machine ceilings its roofline fractions are read against).
 * moe_expert_ffn_between_event: from now on every expert FFN call of this context records `event` (a
 *   hipEvent_t owned by the caller, or NULL to stop) on its stream between its two grouped GEMMs.
 * moe_calibrate_copy: a plain streaming copy of `bytes` (multiple of 16) device bytes with `workgroups`
 *   workgroups of 256 lanes, 16 bytes per lane.
 * moe_calibrate_mfma: a register-resident loop of `iters` x 8 bf16 MFMAs (32x32x16) per wavefront, four
 *   wavefronts per workgroup, on operand bit patterns read once from `operands` (>= 393216 bytes);
 *   2 * 32*32*16 * 8 * iters * 4 * workgroups flop; `sink` receives nothing in practice. */
int moe_expert_ffn_between_event(moe_ctx* ctx, void* event);
int moe_calibrate_copy(void* dst, const void* src, size_t bytes, int32_t workgroups, void* stream);
int moe_calibrate_mfma(const void* operands, float* sink, int32_t iters, int32_t workgroups, void* stream);

/* Combine + scale + cache blend (Algorithm 1 combine/scale; Algorithm 4 "reuse stale h"):
 *   y_i = sum_{j=0..k-1} s*_ij h*_ij   accumulated in float in slot order,
 * where a refreshed pair takes h_packed[inv[p]] and scores[p] and writes both through to
 * H_cache[p] / S_cache[p] (when caches are given), and a reused pair takes H_cache[p] and
 * S_cache[p] (or scores[p] if use_fresh_scores).  The cache is keyed by (token, slot): a change of
 * expert_idx[i][j] on a reused pair is not detected, as with a persistent combine buffer.
 *   in : h_packed[R][d], inv[T*k], scores[T][k], mask[T][k] or NULL (= every pair refreshed).
 *        h_packed may be NULL when caches are given and the shape has no shared experts: the rows of the
 *        refreshed pairs are then expected in H_cache already (moe_expert_ffn_commit put them there),
 *        every row is read from H_cache and only the scores are written through
 *   io : H_cache[T][k][d] (dtype) and S_cache[T][k] float, or both NULL when mask is NULL
 *   out: y[T][d] (dtype)
 * A non-NULL mask with a NULL cache returns MOE_ERR_CACHE_COLD; whether a given cache has been
 * filled by an earlier full refresh is the caller's responsibility. */
int moe_combine(moe_ctx* ctx, const void* h_packed, const int32_t* inv, const float* scores,
                const uint8_t* mask, int32_t T, void* H_cache, float* S_cache,
                int32_t use_fresh_scores, void* y, void* stream);

/* Segment table of an expert-parallel receive buffer (expert-parallelism figure: each device
 * holds a subset of the experts and receives the rows routed to them from every rank).
 * The buffer is ordered [source rank][local expert]; segment g = src*E_loc + e_loc has
 * recv_counts[g] rows and runs on local expert e_loc.
 *   in : recv_counts[W*E_loc] (device)      out: seg_offsets[W*E_loc+1], seg_expert[W*E_loc] */
int moe_ep_segments(moe_ctx* ctx, const int32_t* recv_counts, int32_t W, int32_t E_loc,
                    int32_t* seg_offsets, int32_t* seg_expert, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DICE_MOE_H */
