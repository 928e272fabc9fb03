/*
 * a3.h - C ABI of the per-layer A^3 KV-cache fusion path (arXiv 2511.17560) for one MI355X.
 *
 * The method (section "Attention-Aware Accurate Fusion") fuses per-chunk K/V caches that
 * were precomputed chunk by chunk (Eq. 1) into the cache of the concatenated prompt
 * X = (S, D_1 .. D_k, Q).  Per layer it
 *   1. recovers positions: keys are re-rotated to their position in X        (Eq. 2)
 *   2. scores every context token by the attention the question pays to it    (Eq. 3, first line)
 *   3. keeps the top p = r*n tokens                                           (Eq. 3, second line)
 *   4. recomputes Q/K/V of those tokens and of the question, attends over the
 *      fused cache                                                            (Eq. 4, Eq. 5)
 *   5. writes the fresh K/V back into the fused cache                         (Eq. 5, middle lines)
 *
 * Conventions shared by every entry point
 *   - Pointers named in a3_layout and every tensor / index argument are DEVICE pointers unless
 *     stated otherwise; the a3_layout struct itself lives in HOST memory.
 *   - Everything is allocated and freed by the caller.  The library allocates nothing and only
 *     enqueues kernels on `stream` (a hipStream_t, NULL = the null stream).  No call synchronises
 *     with the host or copies between host and device.  The only state kept between calls is
 *     set-up that is done once per process and device (kernel attributes, the tuning knobs
 *     listed at the end of this header, the address of a3_question_scores_noalloc's scratch array).
 *   - Tensors are dense row-major.  "packed rows": requests back to back, each request being
 *     its context chunks followed by its question tokens.  T = total_tokens.
 *       hidden            [T, hidden]
 *       K / V caches      [T, n_kv_heads, head_dim]
 *       Q / outputs       [n, n_q_heads, head_dim]
 *     Element type is layout->dtype (A3_BF16: bfloat16, A3_F32: float) for all of them.
 *     Every tensor base pointer must be 16-byte aligned.
 *   - Return value: A3_OK or a negative a3_status.  Argument errors are found on the host before
 *     anything is launched (message via a3_last_error()); a failed launch gives A3_ERR_HIP.
 *     Contents of device index arrays cannot be checked on the host: they are preconditions.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point atomics).
 *   - Supported shapes: head_dim 64 or 128, n_q_heads a multiple of n_kv_heads,
 *     hidden a multiple of 32; A3_BF16 additionally needs head_dim 128 and hidden a multiple
 *     of 64 (the MFMA kernels).
 */
#ifndef A3_H
#define A3_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  A3_OK = 0,
  A3_ERR_INVALID_ARG = -1,
  A3_ERR_UNSUPPORTED = -2,
  A3_ERR_WORKSPACE = -3,
  A3_ERR_HIP = -4,
  A3_ERR_IO = -5
} a3_status;

typedef enum { A3_F32 = 0, A3_BF16 = 1 } a3_dtype;

/* Which coordinates form a rotated pair.  INTERLEAVED = (2i, 2i+1), the block-diagonal matrix
 * printed in section "Position Recovery"; HALF = (i, i + head_dim/2). */
typedef enum { A3_ROPE_INTERLEAVED = 0, A3_ROPE_HALF = 1 } a3_rope;
typedef enum { A3_POOL_MAX = 0, A3_POOL_AVG = 1 } a3_pool;

typedef struct a3_layout {
  /* ---- model (host scalars) ---- */
  int dtype;            /* a3_dtype */
  int n_q_heads;
  int n_kv_heads;
  int head_dim;
  int hidden;
  int rope_layout;      /* a3_rope */
  double rope_base;     /* theta_i = rope_base^(-2i/head_dim) */
  float sm_scale;       /* softmax scale; 0 means 1/sqrt(head_dim) */
  /* ---- batch (host scalars) ---- */
  int n_req;            /* requests in the batch */
  int n_chunks;         /* context chunks over all requests */
  int total_tokens;     /* T */
  int max_ctx_len;      /* max over requests of the context length  */
  int max_q_len;        /* max over requests of the question length */
  /* ---- batch (device int32 arrays, caller fills them) ---- */
  const int *seg_start;   /* [n_req+1] packed row of each request's first token; seg_start[n_req] = T */
  const int *ctx_len;     /* [n_req] context tokens of the request (its chunks, back to back) */
  const int *q_len;       /* [n_req] question tokens; seg_start[r+1]-seg_start[r] = ctx_len[r]+q_len[r] */
  const int *chunk_start; /* [n_chunks] packed row of the chunk's first token, strictly ascending */
  const int *chunk_len;   /* [n_chunks] */
  const int *chunk_delta; /* [n_chunks] position of the chunk's first token inside its request:
                             the amount its keys are rotated by in a3_rope_realign */
  /* ---- derived tables (device, caller allocates, a3_layout_prepare fills) ---- */
  int *tok_pos;           /* [T] position of the packed row inside its request */
  int *tok_req;           /* [T] request of the packed row */
  int *tok_chunk;         /* [T] chunk of a context row, -1 for a question row */
  int *q_start;           /* [n_req+1] exclusive prefix sum of q_len: first row of the request in a
                             [sum q_len, ...] question tensor */
  float *rope_chunk_cs;   /* [n_chunks, head_dim/2, 2] (cos, sin) of chunk_delta * theta_i */
  float *rope_pos_cs;     /* [max_ctx_len+max_q_len, head_dim/2, 2] (cos, sin) of p * theta_i */
} a3_layout;

/* Bytes of workspace that a3_question_scores / a3_topk_select / a3_fused_attention may need for
 * this layout when at most max_active_rows rows are active.  Host call, no GPU work. */
size_t a3_workspace_bytes(const a3_layout *layout, int max_active_rows);

/* Fills tok_pos, tok_req, tok_chunk, q_start and both RoPE tables (angles formed and evaluated in
 * double precision, stored as float).  Once per batch of requests; layer independent. */
a3_status a3_layout_prepare(const a3_layout *layout, void *stream);

/* Step 1, Eq. 2 (position recovery).  The cached keys carry RoPE of their chunk-local
 * position; every context key of chunk c is rotated further by chunk_delta[c] so that it
 * carries RoPE of its position in the concatenated prompt.  V is not touched.
 * k_cat, k_fused: [T, n_kv_heads, head_dim].  k_fused may alias k_cat (in place); otherwise
 * they must not overlap, and the question rows of k_fused are left unwritten. */
a3_status a3_rope_realign(const a3_layout *layout, const void *k_cat, void *k_fused, void *stream);

/* Step 2, Eq. 3 first line.  scores[t] = sum over query heads hq and question tokens j of
 * softmax_t(q_{j,hq} . k'_{t, hq / (n_q_heads/n_kv_heads)} * sm_scale), the softmax taken over
 * the context keys of the token's own request.  q_question: [sum q_len, n_q_heads, head_dim]
 * in request order (RoPE already applied); k_fused: realigned cache; scores: float [T],
 * question rows are set to -inf.  ws: at least a3_workspace_bytes() bytes. */
a3_status a3_question_scores(const a3_layout *layout, const void *q_question, const void *k_fused,
                             float *scores, void *ws, size_t ws_bytes, void *stream);

/* a3_question_scores for callers that cannot allocate device memory or hand over a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the
 * workspace), same kernels, bit-identical scores.  The scratch memory the step needs lives in a fixed array of
 * A3_SCORES_SCRATCH_BYTES inside the library's device image (each GPU the library runs on holds one until the
 * process ends); the call allocates and frees nothing.  A batch that needs more (the need grows with
 * n_req * max_q_len * n_q_heads * max_ctx_len / 256 and with n_kv_heads * total_tokens; the 16K-context
 * Llama-3-8B layer takes 1.6 MB, the 32K-context Qwen2.5-7B layer 4.4 MB) is refused with A3_ERR_WORKSPACE
 * before anything is launched.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, different threads) race; calls on one stream are ordered and safe. */
#define A3_SCORES_SCRATCH_BYTES (8u << 20)
a3_status a3_question_scores_noalloc(const a3_layout *layout, const void *q_question, const void *k_fused,
                                     float *scores, void *stream);

/* Steps 1 and 2 in one call: Eq. 2 followed by Eq. 3, first line.  Same results as a3_rope_realign
 * (k_cat -> k_fused, bit for bit) followed by a3_question_scores on k_fused; on the bf16 path the first
 * scoring pass does the rotation itself, so the stale cache is read once instead of the realigned cache
 * being written, then read.  k_cat: keys at chunk-local positions [T, n_kv_heads, head_dim]; k_fused: same
 * shape, may be k_cat itself (in place), otherwise no overlap; as with a3_rope_realign only context rows
 * are written.  Other arguments and errors as for a3_question_scores. */
a3_status a3_realign_scores(const a3_layout *layout, const void *q_question, const void *k_cat, void *k_fused,
                            float *scores, void *ws, size_t ws_bytes, void *stream);

/* Eq. 3, p = r * n: the number of context tokens of a request that are recomputed, n = n_ctx its context length
 * (question tokens are always recomputed and are no candidates), r = ratio_num / ratio_den in [0, 1], rounded down
 * in integer arithmetic.  Host only; -1 on a bad argument.  The caller sums these into sel_start. */
int a3_recompute_count(int n_ctx, int ratio_num, int ratio_den);

/* Step 3, Eq. 3 second line (Re = top_p(s)).  For request r the k_r = sel_start[r+1] -
 * sel_start[r] context rows with the largest scores; equal scores go to the lowest row;
 * sel_idx[sel_start[r] .. sel_start[r+1]) receives packed rows in ascending order.
 * scores: float [T]; sel_start: device int32 [n_req+1], sel_start[0] = 0, k_r <= ctx_len[r];
 * total_k = sel_start[n_req] (host value); sel_idx: device int32 [total_k].
 * NaN scores are not supported. */
a3_status a3_topk_select(const a3_layout *layout, const float *scores, const int *sel_start,
                         int total_k, int *sel_idx, void *ws, size_t ws_bytes, void *stream);

/* Step 4 (projection part), Eq. 5 first lines.  For each listed packed row t:
 *   Q = RoPE_p(x_t Wq^T + bq),  K = RoPE_p(x_t Wk^T + bk),  V = x_t Wv^T + bv,   p = tok_pos[t].
 * hidden: [T, hidden]; row_idx: device int32 [n_rows] (NULL = rows 0..n_rows-1);
 * wq: [n_q_heads*head_dim, hidden], wk, wv: [n_kv_heads*head_dim, hidden] (row-major [out, in]);
 * bq, bk, bv: [out] or NULL.  q_out: [n_rows, n_q_heads, head_dim], k_out, v_out:
 * [n_rows, n_kv_heads, head_dim], compact in list order; each may be NULL to skip it.
 * Accumulation and RoPE in float, one rounding to the storage type on store. */
a3_status a3_selected_qkv_proj(const a3_layout *layout, const void *hidden, const int *row_idx, int n_rows,
                               const void *wq, const void *wk, const void *wv,
                               const void *bq, const void *bk, const void *bv,
                               void *q_out, void *k_out, void *v_out, void *stream);

/* Steps 4 (projection part) and 5 in one call, Eq. 5 first three lines: as a3_selected_qkv_proj, but
 * K and V of listed row i are written straight into the caches at packed row row_idx[i]
 * (k_fused[row_idx[i]] <- K_i, v_fused[row_idx[i]] <- V_i; row_idx NULL means row i); Q stays compact
 * in q_out.  k_fused, v_fused: [T, n_kv_heads, head_dim]; each of the three outputs may be NULL.
 * Saves the round trip of the fresh K/V through a compact buffer and the a3_kv_scatter launch. */
a3_status a3_selected_qkv_proj_scatter(const a3_layout *layout, const void *hidden, const int *row_idx,
                                       int n_rows, const void *wq, const void *wk, const void *wv,
                                       const void *bq, const void *bk, const void *bv,
                                       void *q_out, void *k_fused, void *v_fused, void *stream);

/* Step 5, Eq. 5 middle lines.  k_fused[row_idx[i]] <- k_new[i], v_fused[row_idx[i]] <- v_new[i].
 * k_new, v_new: [n_rows, n_kv_heads, head_dim]; row_idx: device int32 [n_rows], no duplicates.
 * Must be enqueued before a3_fused_attention on the same stream: attention reads the updated rows. */
a3_status a3_kv_scatter(const a3_layout *layout, const void *k_new, const void *v_new, const int *row_idx,
                        int n_rows, void *k_fused, void *v_fused, void *stream);

/* Step 4 (attention part), Eq. 4 and Eq. 5 last line.  For each active row i at packed row
 * t = act_idx[i]:  out[i, hq] = softmax(q_act[i, hq] . K'[u, hq/G] * sm_scale) V[u, hq/G] over the
 * packed rows u of the same request with u <= t (causal by global position, the row itself included).
 * q_act, out: [n_act, n_q_heads, head_dim]; act_idx: device int32 [n_act], strictly ascending.
 * ws: at least a3_workspace_bytes(layout, n_act) bytes. */
a3_status a3_fused_attention(const a3_layout *layout, const void *q_act, const int *act_idx, int n_act,
                             const void *k_fused, const void *v_fused, void *out,
                             void *ws, size_t ws_bytes, void *stream);

/* The same step in two calls.  How a3_fused_attention divides its work among the compute units depends only
 * on the list of active rows, so it can be laid out as soon as that list exists: a3_attention_plan writes the
 * layout into ws (one small kernel), a3_fused_attention_planned then attends with it.  Between the two calls
 * nothing else may write ws; the arguments they share must be the same; stream order (or an event) must put the
 * plan first.  Together they give what a3_fused_attention gives, bit for bit.  a3_fused_attention_planned leaves
 * the plan as it is: further calls with the same act_idx and ws (the layers of a stack whose active rows stay the
 * same) may reuse it. */
a3_status a3_attention_plan(const a3_layout *layout, const int *act_idx, int n_act, void *ws, size_t ws_bytes,
                            void *stream);
a3_status a3_fused_attention_planned(const a3_layout *layout, const void *q_act, const int *act_idx, int n_act,
                                     const void *k_fused, const void *v_fused, void *out,
                                     void *ws, size_t ws_bytes, void *stream);

/* a3_fused_attention_planned for measurements: ev_main_begin / ev_main_end are hipEvent_t handles the caller created
 * (either may be NULL); they are recorded on the stream right before and right after the main attention kernel, so
 * their distance is that kernel's duration alone (the small kernel that merges partial results runs after the
 * second one).  Everything else as a3_fused_attention_planned. */
a3_status a3_fused_attention_planned_events(const a3_layout *layout, const void *q_act, const int *act_idx, int n_act,
                                            const void *k_fused, const void *v_fused, void *out, void *ws,
                                            size_t ws_bytes, void *stream, void *ev_main_begin, void *ev_main_end);

/* Step 3, the row list [Re, Q] and the layout of the attention's work in one call (Eq. 3 second line; Eq. 4 /
 * Eq. 5 act on the rows [Re, Q]): what a3_topk_select (-> sel_idx), a3_active_rows (-> act_idx) and
 * a3_attention_plan (-> ws) give when called one after the other, bit for bit.  For a batch of one request it is a
 * single launch: the workgroup that ranks the scores also writes the row list and the plan.  sel_idx: device
 * int32 [total_k]; in a batch of one request it may be act_idx itself (the selection is the head of the row
 * list).  act_idx: device int32 [n_act], n_act = total_k + sum q_len.  ws: at least
 * a3_workspace_bytes(layout, n_act) bytes; a3_fused_attention_planned with the same act_idx, n_act and ws follows
 * (nothing else may write ws in between). */
a3_status a3_topk_select_plan(const a3_layout *layout, const float *scores, const int *sel_start, int total_k,
                              int *sel_idx, int n_act, int *act_idx, void *ws, size_t ws_bytes, void *stream);

/* Helper between steps 3 and 4: the active rows [Re, Q] of Eq. 4 / Eq. 5 in ascending packed order.
 * For request r, act_idx receives its k_r selected rows followed by its q_len[r] question rows, at
 * offset sel_start[r] + q_start[r].  sel_idx: device int32 [total_k] as written by a3_topk_select;
 * act_idx: device int32 [n_act], n_act = total_k + sum q_len (host value, checked against nothing on
 * the device: it only sizes the launch). */
a3_status a3_active_rows(const a3_layout *layout, const int *sel_idx, const int *sel_start, int n_act,
                         int *act_idx, void *stream);

/* ---- the layer stack around the hot path (Eq. 5, first line: X_l = H(O_{l-1})) -------------------------
 *
 * H(.) takes the attention output of a layer to the input of the next one.  The paper gives it as the
 * layer normalisation and feed-forward network applied to the attention output; taken here as the
 * pre-norm block of the model families it evaluates:
 *     r1 = r0 + O Wo^T,   r2 = r1 + (silu(n1 Wg^T) * (n1 Wu^T)) Wd^T  with n1 = RMSNorm(r1; g_post),
 *     x' = RMSNorm(r2; g_next),        RMSNorm(x; g) = g * x / sqrt(mean(x^2) + eps).
 * All weights are device pointers in the layout's dtype, [out, in] row-major, 16-byte aligned; the
 * caller owns them. */
typedef struct a3_block_weights {
  const void *wo;      /* [hidden, n_q_heads * head_dim] */
  const void *g_post;  /* [hidden]  norm in front of the MLP */
  const void *w_gate;  /* [ffn, hidden] */
  const void *w_up;    /* [ffn, hidden] */
  const void *w_down;  /* [hidden, ffn] */
  const void *g_next;  /* [hidden]  input norm of the next block, or the final norm */
  int ffn;
  float eps;
} a3_block_weights;

/* Bytes of workspace a3_block_tail needs for n_rows rows (host only; 0 on a bad argument). */
size_t a3_block_tail_ws_bytes(const a3_layout *layout, int ffn, int n_rows);

/* H(.) for the active rows.  attn_out: [n_act, n_q_heads, head_dim] as written by a3_fused_attention;
 * act_idx: device int32 [n_act], no duplicates (NULL: rows 0 .. n_act-1).  resid: [total_tokens, hidden],
 * the residual stream; its rows act_idx are read (r0) and overwritten (r2).  hidden_next:
 * [total_tokens, hidden]; its rows act_idx receive x'.  Other rows of both are left alone.
 * bf16 needs hidden % 128 == 0 and ffn % 64 == 0.  Errors: A3_ERR_INVALID_ARG, A3_ERR_UNSUPPORTED,
 * A3_ERR_WORKSPACE before anything is launched. */
a3_status a3_block_tail(const a3_layout *layout, const void *attn_out, const int *act_idx, int n_act,
                        const a3_block_weights *w, void *resid, void *hidden_next,
                        void *ws, size_t ws_bytes, void *stream);

/* RMSNorm of listed rows (the input norm of block 0, in front of the first projection):
 * out[row_idx[i]] = g * x[row_idx[i]] / sqrt(mean(x[row_idx[i]]^2) + eps), x and out [total_tokens, hidden]
 * (may be the same buffer); row_idx NULL: rows 0 .. n_rows-1. */
a3_status a3_rms_norm(const a3_layout *layout, const void *x, const int *row_idx, int n_rows, const void *g,
                      float eps, void *out, void *stream);

/* ---- variants of the selection score and the eviction extension (Method, "Extention") -----------------
 *
 * Eq. 3, first line, with the softmax of a question token taken over every key it sees: the context keys of
 * its request and the question keys up to itself (the literal reading of the equation's denominator;
 * a3_question_scores normalises over the context keys only).  Same arguments as a3_question_scores; the
 * question rows of k_fused must hold the question's keys of this layer. */
a3_status a3_question_scores_causal(const a3_layout *layout, const void *q_question, const void *k_fused,
                                    float *scores, void *ws, size_t ws_bytes, void *stream);

/* Extension, ranking step: votes[g, t] = sum over the query heads of KV head g and over the question tokens
 * of the attention weight context row t receives (softmax over everything the question token sees, as
 * above).  votes: float [n_kv_heads, total_tokens]; entries of question rows are not written.
 * ws: at least a3_workspace_bytes(layout, 0) bytes. */
a3_status a3_window_votes(const a3_layout *layout, const void *q_question, const void *k_fused, float *votes,
                          void *ws, size_t ws_bytes, void *stream);

/* Extension, retention step.  For request r and KV head g, keep_idx[g, keep_start[r] .. keep_start[r+1])
 * receives, in ascending packed-row order: the first sys_len[r] context rows (system prompt), the
 * budget_r = keep_start[r+1] - keep_start[r] - sys_len[r] - q_len[r] best other context rows by votes[g]
 * (ties to the lowest row), and the q_len[r] question rows.  The caller sizes keep_start from the capacity C:
 * budget_r = min(max(C - sys_len[r] - q_len[r], 0), ctx_len[r] - sys_len[r]).
 * votes: float [n_kv_heads, total_tokens]; sys_len: device int32 [n_req]; keep_start: device int32
 * [n_req+1]; total_keep = keep_start[n_req] (host value); keep_idx: device int32 [n_kv_heads, total_keep].
 * pool_width > 1 first smooths the votes along the context rows of each request (odd width <= 63;
 * A3_POOL_MAX, or A3_POOL_AVG with zero padding) into ws (a3_evict_ws_bytes(layout) bytes). */
size_t a3_evict_ws_bytes(const a3_layout *layout);
a3_status a3_evict_select(const a3_layout *layout, const float *votes, const int *sys_len, const int *keep_start,
                          int total_keep, int pool_width, int pool_mode, int *keep_idx,
                          void *ws, size_t ws_bytes, void *stream);

/* Extension, the eviction itself: k_out[slot, g] = k_fused[keep_idx[g, slot], g], same for V.
 * k_out, v_out: [total_keep, n_kv_heads, head_dim]. */
a3_status a3_evict_compact(const a3_layout *layout, const void *k_fused, const void *v_fused, const int *keep_idx,
                           int total_keep, void *k_out, void *v_out, void *stream);

/* ---- alternative producers of the recompute list Re (Experiments, "Baselines"): they replace steps 2-3, the
 * lists feed steps 4-5 unchanged ---------------------------------------------------------------------------
 *
 * Largest value deviation: scores[t] = sum over KV heads and coordinates of (v_true[t] - v_cat[t])^2 for
 * context rows, -inf for question rows; a3_topk_select then takes the top p.  v_true, v_cat:
 * [total_tokens, n_kv_heads, head_dim] (v_true from a V-only a3_selected_qkv_proj over all rows). */
a3_status a3_value_deviation_scores(const a3_layout *layout, const void *v_true, const void *v_cat, float *scores,
                                    void *stream);

/* Chunk edges: for request r, sel_idx[sel_start[r] .. sel_start[r+1]) receives, ascending, the first n_head
 * and the last n_tail rows of each of its chunks (a chunk of at most n_head + n_tail rows: all its rows).
 * The caller sizes sel_start: request r holds sum over its chunks of min(chunk_len, n_head + n_tail) rows;
 * total_k = sel_start[n_req] (host value). */
a3_status a3_select_chunk_edges(const a3_layout *layout, int n_head, int n_tail, const int *sel_start, int total_k,
                                int *sel_idx, void *stream);
/* The sel_start that rule needs, from HOST copies of the layout's arrays: sel_start[r+1] - sel_start[r] = sum over the
 * chunks of request r of min(chunk_len, n_head + n_tail).  sel_start: host int32 [n_req + 1].  Host only. */
a3_status a3_chunk_edge_sel_start(int n_req, const int *seg_start, const int *ctx_len, int n_chunks,
                                  const int *chunk_start, const int *chunk_len, int n_head, int n_tail, int *sel_start);

/* ---- chunk-cache staging (Eq. 1's per-chunk K/V store lives outside the GPU; the paper names loading it as
 * the method's limitation) ---------------------------------------------------------------------------------
 *
 * Copies one layer's chunk blocks from HOST memory into their packed slots of the concatenated caches:
 * rows [chunk_start_host[c], + chunk_len_host[c]) of k_cat / v_cat receive host_k[c] / host_v[c], each a
 * contiguous [chunk_len, n_kv_heads, head_dim] block in the layout's dtype.  chunk_start_host and
 * chunk_len_host are HOST arrays (the layout's own are device pointers); host_k / host_v are host arrays of
 * n_chunks HOST pointers; k_cat, v_cat are device pointers.  The copies are enqueued on `stream` and are
 * asynchronous when the host blocks are pinned (hipHostMalloc); the caller keeps the blocks alive until the
 * stream has passed them.  Nothing is allocated.  Errors: A3_ERR_INVALID_ARG (before any copy is enqueued),
 * A3_ERR_HIP. */
a3_status a3_chunk_cache_load(const a3_layout *layout, const int *chunk_start_host, const int *chunk_len_host,
                              int n_chunks, const void *const *host_k, const void *const *host_v,
                              void *k_cat, void *v_cat, void *stream);

/* The chunk store itself sits on persistent storage (Eq. 1; the paper names loading it as the method's limitation).
 * a3_chunk_file_read brings one layer's blocks from already opened files into HOST staging buffers, from which
 * a3_chunk_cache_load / a3_chunk_cache_load_q8 copy them on (asynchronously if the buffers are pinned): block c is
 * n_bytes[c] bytes at file_offset[c] of the descriptor fds[c], read into host_dst[c].  All arguments are host
 * arrays of n_blocks entries.  Positional reads (the descriptors' own offsets are not used or moved), continued
 * after short reads, spread block by block over up to n_threads (1..16) threads; the call returns when every block
 * is in memory.  No GPU call, nothing allocated beyond the threads.  Errors: A3_ERR_INVALID_ARG before any read;
 * A3_ERR_IO when a read fails or a file ends inside a block (a3_last_error() names the block). */
a3_status a3_chunk_file_read(int n_blocks, const int *fds, const long long *file_offset, const size_t *n_bytes,
                             void *const *host_dst, int n_threads);

/* ---- 8-bit form of the chunk caches (the paper fixes no format and calls cache quantisation orthogonal; it
 * halves what the staging above has to move) -----------------------------------------------------------------
 *
 * One packed row of one layer is one record of a3_q8_row_bytes(layout) = n_kv_heads * (2 * head_dim + 8) bytes:
 *     [ K codes: n_kv_heads * head_dim int8 | V codes: the same | K scales: n_kv_heads float32 | V scales ],
 * x = code * scale per row and KV head (symmetric).  A chunk's rows of both caches are one contiguous block.
 * cache_q8 is [total_tokens] records, device, 16-byte aligned.
 *
 * a3_quantize_q8: the quantiser, run once when a chunk's caches are produced: k, v [total_tokens, n_kv_heads,
 * head_dim] in the layout's dtype (finite values) -> records; the scale is the float32 rounding of max|x| / 127,
 * the code the quotient x / scale rounded half to even, both taken in float64; a row of zeros gets scale 0 and
 * codes 0.
 * a3_rope_realign_q8: step 1 (Eq. 2) on the dequantised keys, and the values, in one kernel: k_fused receives,
 * for context rows, the dequantised key turned by its chunk's offset, for question rows the dequantised key;
 * v_fused receives the dequantised value; one rounding to the layout's dtype each.  Either output may be NULL.
 * a3_chunk_cache_load_q8: as a3_chunk_cache_load, one host block of chunk_len[c] records and one copy per
 * chunk. */
size_t a3_q8_row_bytes(const a3_layout *layout);
a3_status a3_quantize_q8(const a3_layout *layout, const void *k, const void *v, void *cache_q8, void *stream);
a3_status a3_rope_realign_q8(const a3_layout *layout, const void *cache_q8, void *k_fused, void *v_fused,
                             void *stream);
a3_status a3_chunk_cache_load_q8(const a3_layout *layout, const int *chunk_start_host, const int *chunk_len_host,
                                 int n_chunks, const void *const *host_q8, void *cache_q8, void *stream);

/* ---- tuning values (for tests and measurements; the defaults are what the library picks by itself) -----------
 * Process-wide integers, read when a call is made; value < 0 restores the library's own choice.  Names:
 *   "attn_wgs"        workgroups (shares of the work) per KV head in a3_fused_attention, 1 .. 1024
 *   "attn_item_cost"  start-up cost of a row tile, in 64-key steps, that the shares are balanced with, 0 .. 64
 *   "proj_ntw"        row-tile width (2, 3, 4: 128, 192, 256 rows) of the projection GEMM; set, it also sends
 *                     calls with few rows to that kernel instead of the weight-streaming one
 *   "proj_k64"        0: the projection's main loop on 64-byte instead of 128-byte row pieces
 *   "gemm_tb", "gemm_k64"   the same two for the GEMMs of a3_block_tail
 * A value must not change between a3_attention_plan and the a3_fused_attention_planned calls that use its plan:
 * if "attn_wgs" does, the plan lies elsewhere in the workspace, the kernels of the planned call notice (the
 * plan records the value it was made with at a fixed place) and leave `out` untouched.
 * Host only; A3_ERR_INVALID_ARG for an unknown name. */
a3_status a3_set_tuning(const char *name, int value);

const char *a3_strerror(a3_status status);
/* Text of the last error raised on the calling thread ("" if none). */
const char *a3_last_error(void);
int a3_version(void);

#ifdef __cplusplus
}
#endif
#endif /* A3_H */
