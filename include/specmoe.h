/*
 * specmoe.h - C ABI of the MI355X (gfx950) MoE verification layer.
 *
 * The library computes, for one Mixture-of-Experts block, what the target model has to
 * compute when it verifies a batch of speculative draft tokens (SpecMoE, arxiv 2604.10152):
 * B sequences with gamma draft tokens each are scored in one parallel pass (Sec. 2.2
 * "Algorithm", Fig. 4), so the block sees T = B*(gamma+1) tokens; its gate picks the top-K of
 * E experts per token and only the picked experts run (Sec. 2.1, Fig. 1b); afterwards the
 * greedy rule keeps the longest prefix of drafts that equals the target's own tokens and
 * appends one target token (Sec. 2.2 Fig. 4 caption; Sec. 4 "SpecMoE configuration").
 *
 * Conventions shared by every entry point
 *  - Every pointer except `stream` is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or keeps a pointer after the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; they never synchronise.
 *  - All matrices are dense row-major.  `dtype` selects the element type of activations and
 *    weights (x, w_*, x_perm, y_perm, out, gain): SPECMOE_F32 = IEEE binary32,
 *    SPECMOE_BF16 = bfloat16.  Gate weights are always float, indices always int32_t.
 *  - Arguments are validated on the host before anything is enqueued.  A non-zero return
 *    value (specmoe_status) means nothing was enqueued.  Sizes of zero tokens / sequences
 *    are legal and enqueue nothing (moe_permute still writes expert_offsets).
 *  - bf16 mode requires d_model % 64 == 0 and d_ff % 64 == 0; fp32 mode has no such limit.
 *  - 1 <= k <= E <= SPECMOE_MAX_EXPERTS, k <= SPECMOE_MAX_TOPK.
 *  - Results are deterministic: no floating-point atomics anywhere.
 */
#ifndef SPECMOE_H_
#define SPECMOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPECMOE_OK = 0,
    SPECMOE_ERR_NULL = 1,       /* a required pointer is NULL                       */
    SPECMOE_ERR_SHAPE = 2,      /* negative size, k > E, unsupported divisibility   */
    SPECMOE_ERR_DTYPE = 3,      /* dtype is neither SPECMOE_F32 nor SPECMOE_BF16     */
    SPECMOE_ERR_WORKSPACE = 4,  /* workspace smaller than the query function says    */
    SPECMOE_ERR_DEVICE = 5      /* the HIP runtime refused the launch                */
} specmoe_status;

typedef enum { SPECMOE_F32 = 0, SPECMOE_BF16 = 1 } specmoe_dtype;

#define SPECMOE_MAX_EXPERTS 1024
#define SPECMOE_MAX_TOPK 64
#define SPECMOE_MAX_GAMMA 64     /* draft tokens per sequence in spec_accept_sample */

/* Gate of one MoE block (Sec. 2.1: "the gate selects the top-K experts per token").
 *   logits l[t,e] = router_bias[e] + sum_j x[t,j] * w_router[e,j], accumulated in fp64;
 *   topk_idx[t,0..k-1] = the k experts with the largest LOGITS, slot order = descending
 *   logit, equal logits -> lower expert id first;
 *   topk_w[t,s] = softmax(l[t,:])[topk_idx[t,s]], divided by sum_s topk_w[t,s] if renorm != 0.
 * x [T,d_model], w_router [E,d_model] in `dtype`; router_bias [E] float or NULL;
 * topk_idx [T,k] int32; topk_w [T,k] float. */
int moe_route_topk(const void* x, const void* w_router, const float* router_bias,
                   int T, int d_model, int E, int k, int renorm, int dtype,
                   int32_t* topk_idx, float* topk_w, void* stream);

/* Grouping of the P = T*k (token, slot) pairs by expert (Fig. 2: tokens that activate the
 * same expert are served together; Sec. 3.2: per-expert activation counts of the
 * verification pass = expert_offsets[e+1] - expert_offsets[e]).
 *   expert_offsets [E+1]: exclusive prefix sum of the per-expert pair counts;
 *   row_src [P]: sorted row r holds flat pair row_src[r] = t*k + s;
 *   row_of  [P]: inverse map, row_of[t*k+s] = r;
 *   x_perm  [P,d_model]: x_perm[r] = x[row_src[r] / k]  (may be NULL: indices only).
 * The sort is stable: inside an expert rows keep ascending flat pair index.  Every
 * topk_idx value must lie in [0,E); values outside are clamped into the range. */
int moe_permute(const void* x, const int32_t* topk_idx, int T, int d_model, int E, int k,
                int dtype, void* x_perm, int32_t* expert_offsets, int32_t* row_src,
                int32_t* row_of, void* stream);

/* Bytes of scratch moe_grouped_swiglu needs for these sizes (0 on invalid arguments). */
size_t moe_grouped_swiglu_workspace_bytes(int n_rows, int d_model, int d_ff, int E, int dtype);

/* Experts (Sec. 2.1: each expert has the size of the FFN layer; only activated ones run).
 * For every expert e and row r in [expert_offsets[e], expert_offsets[e+1]):
 *   h = silu(x_perm[r] . w_gate[e]^T) * (x_perm[r] . w_up[e]^T),  silu(z) = z/(1+exp(-z))
 *   y_perm[r] = h . w_down[e]^T
 * x_perm, y_perm [n_rows,d_model]; w_gate, w_up [E,d_ff,d_model]; w_down [E,d_model,d_ff];
 * expert_offsets [E+1] non-decreasing with expert_offsets[E] <= n_rows (device memory; it
 * is never read on the host).  bf16 mode: bf16 operands, fp32 accumulation on the matrix
 * cores, h and y_perm each rounded to bf16 once.  fp32 mode: fp32 FMA throughout.
 * `workspace` holds h and must be 256-byte aligned. */
int moe_grouped_swiglu(const void* x_perm, const int32_t* expert_offsets,
                       const void* w_gate, const void* w_up, const void* w_down,
                       int n_rows, int d_model, int d_ff, int E, int dtype,
                       void* y_perm, void* workspace, size_t workspace_bytes, void* stream);

/* moe_grouped_swiglu for callers that cannot allocate device memory or size a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * intermediate h lives in a file-scope device array of the library instead of a caller
 * workspace.  Same kernels and the same results as moe_grouped_swiglu.  The call allocates
 * nothing; n_rows * d_ff * sizeof(element) must not exceed SPECMOE_STATIC_SCRATCH_BYTES
 * (SPECMOE_ERR_WORKSPACE otherwise, nothing launched).  Every GPU the library runs on holds
 * its own copy of the array until the process ends.  All calls on one GPU share it, so calls
 * that overlap in time on one GPU (different streams or threads) race on h; rows [0, n_rows)
 * of h are fully overwritten by every call, nothing has to start at zero. */
#define SPECMOE_STATIC_SCRATCH_BYTES (16u << 20)
int moe_grouped_swiglu_static(const void* x_perm, const int32_t* expert_offsets,
                              const void* w_gate, const void* w_up, const void* w_down,
                              int n_rows, int d_model, int d_ff, int E, int dtype,
                              void* y_perm, void* stream);

/* The two halves of moe_grouped_swiglu as separate calls (same definitions, same kernels):
 *   moe_expert_up_swiglu:  h[r] = silu(x_perm[r] . w_gate[e]^T) * (x_perm[r] . w_up[e]^T)
 *   moe_expert_down:       y_perm[r] = h[r] . w_down[e]^T
 * h is [n_rows,d_ff] in `dtype`.  moe_grouped_swiglu(...) == up into `workspace`, then down. */
int moe_expert_up_swiglu(const void* x_perm, const int32_t* expert_offsets, const void* w_gate,
                         const void* w_up, int n_rows, int d_model, int d_ff, int E, int dtype,
                         void* h, void* stream);
int moe_expert_down(const void* h, const int32_t* expert_offsets, const void* w_down, int n_rows,
                    int d_model, int d_ff, int E, int dtype, void* y_perm, void* stream);

/* moe_expert_up_swiglu with the row gather of moe_permute folded into its loads: row r of the
 * (never materialised) x_perm is x[row_src[r] / k], x being the [T,d_model] token matrix.  Same
 * result as moe_permute(x -> x_perm) followed by moe_expert_up_swiglu(x_perm); call
 * moe_permute with x_perm = NULL to get the indices only.  n_rows <= T*k;
 * T * d_model * sizeof(element) must stay below 4 GiB. */
int moe_expert_up_swiglu_gather(const void* x, const int32_t* row_src, int T, int k,
                                const int32_t* expert_offsets, const void* w_gate,
                                const void* w_up, int n_rows, int d_model, int d_ff, int E,
                                int dtype, void* h, void* stream);

/* Tile-packed operands for the large-batch regime (Sec. 2.2: verification brings hundreds of
 * rows per expert, the expert GEMMs are then bound by the rate at which L2 serves requests;
 * packed operands turn sixteen 64-byte requests into eight 128-byte ones).
 * Layout of a tile-packed bf16 matrix [R, K] (R % 16 == 0, K % 32 == 0; same size as row-major):
 * 1 KB blocks of 16 rows x 32 columns, block (rb, kb) at byte offset (rb * (K/32) + kb) * 1024;
 * inside a block the 16-byte chunk c (columns 8c..8c+7 of the block) of row r is piece number
 * 4*r + (c ^ ((r/2) % 4)).
 *   moe_pack_weights: w [E, n_rows, n_cols] row-major -> w_packed (same shape, every expert's
 *     matrix tile-packed); out of place, w_packed must not overlap w.  One-time work: the
 *     paper's experts are fixed during inference (Sec. 2.1).  bf16 only; n_rows % 16 == 0,
 *     n_cols % 32 == 0.
 *   moe_packed_h_bytes: size of the tile-packed intermediate h for n_rows rows (every expert's
 *     rows padded to whole 16-row blocks: at most n_rows + 16*E rows).
 *   moe_expert_up_swiglu_gather_packed: as moe_expert_up_swiglu_gather (row_src == NULL: x is
 *     x_perm [n_rows, d_model]) with w_gate / w_up tile-packed; writes h tile-packed: row r of
 *     expert e (r counted from expert_offsets[e]) is row 16 * B_e + r of the packed matrix,
 *     B_e = sum over e' < e of ceil(rows(e') / 16); padding rows are written as zeros.
 *     x_packed_workspace (may be NULL): moe_packed_h_bytes(n_rows, d_model, E) bytes of scratch;
 *     if given, the token rows are first gathered into it in the same tile-packed row numbering
 *     (one extra pass over x) so that the activation loads are 1 KB pieces as well.
 *   moe_permute_rows_packed / moe_expert_up_swiglu_packed: the two steps of the call above with a
 *     workspace, as calls of their own (the packed rows are then the caller's buffer: the token
 *     dispatch of Sec. 2.1 written once in the layout the GEMM loads).  moe_permute_rows_packed
 *     gathers x[row_src[r] / k] (row_src == NULL: x[r]) into x_packed, row numbering as for h,
 *     padding rows zero; x 16-byte aligned.  moe_expert_up_swiglu_packed reads such an x_packed
 *     (x_packed_bytes >= moe_packed_h_bytes(n_rows, d_model, E)) and writes h tile-packed
 *     (h_row_major == 0, h_bytes >= moe_packed_h_bytes(n_rows, d_ff, E)) or as the row-major
 *     [n_rows, d_ff] matrix moe_expert_down reads (h_row_major != 0, h_bytes >= n_rows*d_ff*2):
 *     with tens of rows per expert the packed gate/up kernel is ahead of the row-major one while
 *     the row-major down kernels are ahead of the packed one.
 *   moe_expert_down_packed: as moe_expert_down with h and w_down tile-packed; y_perm row-major.
 * Results are identical to the row-major entry points' large-batch kernels (same arithmetic in
 * the same order) where both pick the same tile.  moe_expert_up_swiglu_packed and
 * moe_expert_down_packed choose 320-row tiles from 192 rows per expert on average and 192-row
 * tiles below; moe_expert_up_swiglu_gather_packed without a workspace always uses 320-row tiles.
 * With long contractions (>= 4096) and fewer than about 48 rows per expert the row-major entry
 * points are the faster ones.  bf16 only. */
int moe_pack_weights(const void* w, int E, int n_rows, int n_cols, int dtype, void* w_packed,
                     void* stream);
size_t moe_packed_h_bytes(int n_rows, int d_ff, int E);
int moe_expert_up_swiglu_gather_packed(const void* x, const int32_t* row_src, int T, int k,
                                       const int32_t* expert_offsets, const void* w_gate_packed,
                                       const void* w_up_packed, int n_rows, int d_model, int d_ff,
                                       int E, int dtype, void* h_packed, size_t h_packed_bytes,
                                       void* x_packed_workspace, size_t x_packed_workspace_bytes,
                                       void* stream);
int moe_permute_rows_packed(const void* x, const int32_t* row_src, int T, int k,
                            const int32_t* expert_offsets, int n_rows, int d_model, int E,
                            int dtype, void* x_packed, size_t x_packed_bytes, void* stream);
int moe_expert_up_swiglu_packed(const void* x_packed, size_t x_packed_bytes,
                                const int32_t* expert_offsets, const void* w_gate_packed,
                                const void* w_up_packed, int n_rows, int d_model, int d_ff, int E,
                                int dtype, void* h, size_t h_bytes, int h_row_major, void* stream);
int moe_expert_down_packed(const void* h_packed, const int32_t* expert_offsets,
                           const void* w_down_packed, int n_rows, int d_model, int d_ff, int E,
                           int dtype, void* y_perm, void* stream);

/* Gate-weighted mix of the selected experts' outputs (Sec. 2.1, Fig. 1b):
 *   out[t] = (residual ? residual[t] : 0) + sum_{s<k} topk_w[t,s] * y_perm[row_of[t*k+s]]
 * accumulated in fp32 in slot order, rounded once to `dtype`.  residual [T,d_model] in
 * `dtype` or NULL; out may alias residual. */
int moe_combine(const void* y_perm, const int32_t* row_of, const float* topk_w,
                const void* residual, int T, int d_model, int k, int dtype, void* out,
                void* stream);

/* Greedy verification (Sec. 2.2 Fig. 4; Sec. 4: only drafts that exactly match the target's
 * greedy tokens are accepted).  draft_ids [B,gamma]; target_ids [B,gamma+1], target_ids[b,i]
 * being the target's token for the position draft_ids[b,i] was proposed for and
 * target_ids[b,gamma] the extra token.  n_b = number of leading matches;
 *   accept_len[b] = n_b + 1   (tokens generated this step, in [1,gamma+1]);
 *   out_tokens[b,0..n_b] = target_ids[b,0..n_b], remaining entries -1.   gamma = 0 is legal. */
int spec_accept(const int32_t* draft_ids, const int32_t* target_ids, int B, int gamma,
                int32_t* accept_len, int32_t* out_tokens, void* stream);

/* Temporally hot experts of the block (Sec. 3.2 "Expert replacement policy", Fig. 7 steps 3-4:
 * the experts activated most during this verification pass become the draft experts of the
 * next speculation phase).  counts[e] = expert_offsets[e+1] - expert_offsets[e];
 *   hot_ids[0..n_hot-1] = the n_hot experts with the largest counts, ordered by descending
 *   count, equal counts -> lower expert id first;  hot_counts[s] = counts[hot_ids[s]] (may be
 *   NULL).  0 <= n_hot <= E. */
int moe_hot_experts(const int32_t* expert_offsets, int E, int n_hot, int32_t* hot_ids,
                    int32_t* hot_counts, void* stream);

/* ---- speculation phase: draft experts and the affinity table (Sec. 3.2 "Affinity-based expert
 * selection mechanism", Fig. 8) --------------------------------------------------------------
 *
 * moe_affinity_table: the offline table of pairwise L2 distances between the experts of one
 * block.  An expert's parameters are its three matrices together:
 *   affinity[i,j] = sqrt( |Wg_i-Wg_j|_F^2 + |Wu_i-Wu_j|_F^2 + |Wd_i-Wd_j|_F^2 ),  [E,E] float,
 * exactly symmetric, zero diagonal.  w_gate, w_up [E,d_ff,d_model], w_down [E,d_model,d_ff] as
 * for the expert entry points; d_model*d_ff*sizeof(element) must be a multiple of 16 and the
 * weight pointers 16-byte aligned (else SPECMOE_ERR_SHAPE).  `workspace`: device scratch of at
 * least moe_affinity_table_workspace_bytes(E) bytes, 8-byte aligned, contents irrelevant
 * (SPECMOE_ERR_WORKSPACE if smaller).  Sums are accumulated in fp64 in a fixed order, so the
 * result is deterministic. */
size_t moe_affinity_table_workspace_bytes(int E);
int moe_affinity_table(const void* w_gate, const void* w_up, const void* w_down, int E,
                       int d_model, int d_ff, int dtype, float* affinity, void* workspace,
                       size_t workspace_bytes, void* stream);

/* moe_nearest_draft_expert: for one set of draft (GPU-resident) experts, remap[e] = e if e is a
 * draft expert, otherwise the draft expert d with the smallest affinity[e,d]; equal distances ->
 * lower id.  draft_ids [n_draft] (device, any order, 1 <= n_draft <= E); ids outside [0,E) are
 * ignored.  Typically draft_ids = hot_ids of moe_hot_experts. */
int moe_nearest_draft_expert(const float* affinity, int E, const int32_t* draft_ids, int n_draft,
                             int32_t* remap, void* stream);

/* moe_route_topk_draft: the router of the draft model.  The target's gate is used unchanged
 * (same logits, top-k and gate weights as moe_route_topk); every selected expert e is then
 * replaced by remap[e] (device, [E]), slot by slot, keeping the slot's gate weight.  Two slots
 * of a token may name the same draft expert; moe_permute / moe_combine handle that (the
 * weights add).  All other arguments as moe_route_topk. */
int moe_route_topk_draft(const void* x, const void* w_router, const float* router_bias, int T,
                         int d_model, int E, int k, int renorm, int dtype, const int32_t* remap,
                         int32_t* topk_idx, float* topk_w, void* stream);

/* ---- sampling-based verification (Sec. 6.3: the models without pronounced hotness are verified
 * with the sampling rule of the speculative-decoding method the paper cites, temperature 1) ----
 * draft_ids [B,gamma]; p_draft [B,gamma,V] = the draft model's distribution at each drafted
 * position; p_target [B,gamma+1,V]; u_accept [B,gamma] and u_sample [B]: uniforms in [0,1)
 * supplied by the caller (the result is a deterministic function of the inputs).  All float.
 * Draft i (id x) is kept iff u_accept[b,i]*p_draft[b,i,x] < p_target[b,i,x] (evaluated exactly,
 * in fp64); n_b = number of drafts kept before the first rejection.  If n_b < gamma the token at
 * position n_b is drawn from max(p_target - p_draft, 0) at that position, else from
 * p_target[b,gamma]: the smallest id whose running sum (fp64, ascending ids) exceeds
 * u_sample[b] * total.  accept_len[b] = n_b + 1; out_tokens[b,0..n_b-1] = the kept drafts,
 * out_tokens[b,n_b] = the drawn token, remaining entries -1.  0 <= gamma <= SPECMOE_MAX_GAMMA.
 * A draft id outside [0,V) is rejected. */
int spec_accept_sample(const int32_t* draft_ids, const float* p_draft, const float* p_target,
                       const float* u_accept, const float* u_sample, int B, int gamma, int V,
                       int32_t* accept_len, int32_t* out_tokens, void* stream);

/* Greedy head in front of spec_accept (Sec. 4 "SpecMoE configuration": greedy decoding):
 * tokens[r] = id of the largest of logits[r,0..V-1] ([R,V], `dtype`), lower id on ties.
 * Logits must not contain NaN. */
int spec_greedy_tokens(const void* logits, int R, int V, int dtype, int32_t* tokens,
                       void* stream);

/* Parameter volume of the experts that at least one token activated in this pass (Sec. 2.1
 * "Challenges in MoE model inference", Fig. 3(b): the bytes an offloading system migrates for
 * the block; on this build: the weight bytes the expert kernels read from HBM).
 * out_bytes[0] = #{e : expert_offsets[e+1] > expert_offsets[e]} * bytes_per_expert (device). */
int moe_active_expert_bytes(const int32_t* expert_offsets, int E, long long bytes_per_expert,
                            long long* out_bytes, void* stream);

/* Helper for the multi-layer benchmark configuration (not part of the paper's method):
 * out[t] = x[t] / sqrt(mean_j x[t,j]^2 + eps) * gain, fp32 arithmetic, rounded to `dtype`. */
int moe_rmsnorm(const void* x, const void* gain, int T, int d_model, float eps, int dtype,
                void* out, void* stream);

/* Static description of a status code. */
const char* specmoe_status_string(int status);

/* ABI version of this header (bumped on any signature change). */
int specmoe_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECMOE_H_ */
