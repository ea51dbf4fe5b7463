/*
 * libdapq — DapQ eviction scoring for MI355X (gfx950), C ABI.
 *
 * DapQ ("Where Matters More Than What", Sec. 4) decides which prompt keys to keep before decoding
 * starts: N pseudo queries that carry the RoPE positions of the first N decode steps
 * (L_p .. L_p+N-1, Sec. 4.1) attend to the L_p prompt keys; the attention mass each key receives
 * is summed over the pseudo queries (Sec. 4.2, importance score S(j)), and only the TopK keys per
 * head survive (Sec. 4.2, M_retain); their K/V rows form the compact cache that decoding uses.
 *
 * Conventions for every entry point
 *   - C linkage, plain C types.  Returns DAPQ_OK (0) or a negative DAPQ_ERR_* code;
 *     dapq_last_error() gives a thread-local message for the last failure on this thread.
 *   - Every data pointer is DEVICE memory unless the comment says "host".  The caller owns all
 *     buffers (inputs, outputs, workspace); the library allocates nothing, frees nothing and keeps
 *     no pointer after the call returns.  Inputs are never written.
 *   - Arguments are validated on the host before anything is enqueued; a failing call enqueues
 *     nothing.  Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the call returns without synchronising.
 *   - Calls may be in flight on several streams at once as long as they share no output buffer and no
 *     workspace: a workspace belongs to one call until the work of that call has finished on its stream.
 *   - Results are deterministic: the same inputs give the same bits on every run.
 *   - Every call only launches kernels on `stream` (no memset or copy nodes, no synchronisation), so a sequence
 *     of calls can be recorded into a HIP graph and replayed; counters in the workspace are cleared by the
 *     kernels of each call.  The first call of an entry point on a device also raises its kernels' dynamic-LDS
 *     limits and reads the device's unit count, which is host work: make one ordinary call before capturing.
 *   - bf16 tensors are passed as void* (16-bit patterns).  head_dim must be 128.
 *
 * Tensor layouts (element strides, the last dimension d is contiguous)
 *   Q  pseudo queries, bf16, already rotated to positions L_p+i:
 *        q[layer*q_stride_layer + seq*q_stride_seq + head*q_stride_head + i*q_stride_row + c]
 *   K, V  prompt keys / values, bf16, keys already rotated to their positions:
 *        k[layer*k_stride_layer + seq*k_stride_seq + kv_head*k_stride_head + t*k_stride_token + c]
 *        where t = cu_seqlens[seq] + j is the packed token index of key j of sequence seq
 *        (k_stride_seq comes on top of the packed token offset: 0 for a packed [tokens][heads][d]
 *        layout, g*k_stride_token if g rows that are not part of the batch follow every sequence).
 *   scores / pooled   fp32 [n_layers][n_kv_heads][total_tokens]   (packed token index)
 *   idx     int32 [n_layers][batch][n_kv_heads][budget]   positions j inside the sequence, ascending
 *   count   int32 [n_layers][batch][n_kv_heads]           = min(budget of the sequence, L_p)
 *   k_out, v_out  bf16 [n_layers][batch][n_kv_heads][budget][d]
 */
#ifndef DAPQ_H
#define DAPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DAPQ_OK = 0,
  DAPQ_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, heads not divisible, even pool width ... */
  DAPQ_ERR_UNSUPPORTED = -2, /* head_dim != 128, stride not a multiple of 8 elements, misaligned base */
  DAPQ_ERR_WORKSPACE = -3,   /* workspace smaller than dapq_workspace_bytes() */
  DAPQ_ERR_HIP = -4          /* the HIP runtime refused a launch */
};

typedef struct dapq_shape {
  int32_t n_layers;
  int32_t batch;          /* sequences */
  int32_t n_q_heads;      /* H_q, a multiple of n_kv_heads; query head h belongs to KV head h / (H_q/H_kv) */
  int32_t n_kv_heads;     /* H_kv */
  int32_t head_dim;       /* d_k = 128 */
  int32_t n_pseudo;       /* N pseudo queries per query head (Sec. 4.1) */
  int64_t total_tokens;   /* sum of L_p over the batch */
  const int32_t* cu_seqlens; /* device, [batch+1], cu_seqlens[0] = 0, non-decreasing, last = total_tokens;
                                NULL = every sequence has L_p = total_tokens / batch */
  int64_t k_stride_layer, k_stride_seq, k_stride_head, k_stride_token;
  int64_t v_stride_layer, v_stride_seq, v_stride_head, v_stride_token;
  int64_t q_stride_layer, q_stride_seq, q_stride_head, q_stride_row;
  float scale;            /* 1/sqrt(d_k) (App. C.1: Attention(q,K) = softmax(qK^T/sqrt(d_k))) */
} dapq_shape;

/* Bytes of device workspace dapq_score / dapq_score_stats / dapq_score_accumulate need for this shape
 * (one figure covers all of them).  Returns 0 if the shape is invalid. */
size_t dapq_workspace_bytes(const dapq_shape* shape);

/* Message for the last error returned on the calling thread ("" if none). Host pointer, owned by the library. */
const char* dapq_last_error(void);

/* Sec. 4.1 — position assignment.  Rotates every (row, head) vector of x_in to the absolute
 * position pos[row] with rotary embedding: channel pair c turns by pos * theta^(-2c/head_dim).
 * For the pseudo queries of a prompt of length L_p the caller passes pos = L_p .. L_p+N-1.
 *   x_in, x_out  bf16, element (row, head, c) at row*stride_row + head*stride_head + c; x_out may
 *                equal x_in (in place) but must not otherwise overlap it.
 *   pos          int32 [rows], >= 0.
 *   pairing      0: channel c pairs with c + head_dim/2;  1: channel 2c pairs with 2c+1.
 * Angles and the rotation are evaluated in fp64, the result is rounded to bf16 once (nearest even). */
int dapq_rope_apply(const void* x_in, void* x_out, const int32_t* pos, int64_t rows, int32_t heads,
                    int32_t head_dim, int64_t stride_row, int64_t stride_head, double theta,
                    int32_t pairing, void* stream);

/* Sec. 4.1 (Positions(T_pseudo) = [L_p, ..., L_p+N-1]) with the content choice of Sec. 5.1 (the first m and
 * the last n tokens of the prompt, N = m + n): for every sequence of the batch
 *   token_idx[seq][i]   packed index (cu_seqlens[seq] + j) of the prompt token pseudo token i copies:
 *                       j = i for i < m, j = L_p - n + (i - m) after that; a prompt shorter than m or n
 *                       repeats its first / last token; -1 for an empty prompt
 *   positions[seq][i]   L_p + i, ready for dapq_rope_apply
 * Both device, int32 [batch][n_pseudo]; first_m + last_n must equal shape->n_pseudo.  Sequence lengths are
 * read on the device (cu_seqlens), so a ragged batch needs no host round trip. */
int dapq_pseudo_tokens(const dapq_shape* shape, int32_t first_m, int32_t last_n, int32_t* token_idx,
                       int32_t* positions, void* stream);

/* Sec. 4.1 — the queries of the pseudo tokens.  The model runs the pseudo tokens only to obtain their queries;
 * pseudo token r copies prompt token token_idx[r] (dapq_pseudo_tokens), so for every layer its row of the
 * query projection's input is that token's row, and
 *   q_out[layer][head][r][c] = RoPE_{positions[r]}( bf16( sum_t x[layer][token_idx[r]][t] * w_q[layer][head*head_dim + c][t] ) )
 * with fp32 accumulation, one rounding to bf16 (nearest even) and then the rotation of dapq_rope_apply.
 *   x          device, bf16: the input rows of the query projection (the layer's normalised hidden states),
 *              element (layer, token, t) at layer*x_stride_layer + token*x_stride_token + t; x_stride_layer may
 *              be 0 (one set of rows for all layers); one layer must span less than 4 GiB
 *   token_idx  device, int32 [rows]: packed prompt token each pseudo token copies; a negative entry has no
 *              source and yields a zero query; entries >= total_tokens read as zero rows
 *   w_q        device, bf16: query weights, one row of `hidden` inputs per output feature,
 *              element (layer, f, t) at layer*w_stride_layer + f*w_stride_row + t, f = head*head_dim + c
 *   positions  device, int32 [rows] (L_p + i of the row's sequence), or NULL: no rotation (theta, pairing unused)
 *   q_out      device, bf16, element (layer, head, r, c) at layer*q_stride_layer + head*q_stride_head +
 *              r*q_stride_row + c; with r = seq*N + i this is the Q layout of dapq_score when
 *              q_stride_seq = N*q_stride_row
 *   workspace  device scratch of at least dapq_pseudo_queries_workspace_bytes(desc), 16-byte aligned; may be NULL
 *              when that is 0.  It is needed when the call is too small to fill the chip with one wave per
 *              weight tile (a single layer, say): the hidden axis is then split over several waves whose fp32
 *              sums meet there and are added in a fixed order.
 * hidden must be a multiple of 64, head_dim a multiple of 8 (even), strides multiples of 8 elements, bases
 * 16-byte aligned.  The weight is streamed once per sweep of 64 rows; the kernel is built for the few rows of
 * a pseudo segment (batch * N up to a few hundred), not for prompt-sized products. */
typedef struct dapq_qproj {
  int32_t n_layers;
  int32_t rows;          /* pseudo tokens of all sequences: batch * N */
  int32_t hidden;        /* inputs of the projection */
  int32_t n_q_heads;     /* H_q */
  int32_t head_dim;      /* d_k; the projection has H_q * d_k output features */
  int64_t total_tokens;  /* rows of x per layer */
  int64_t x_stride_layer, x_stride_token;
  int64_t w_stride_layer, w_stride_row;
  int64_t q_stride_layer, q_stride_head, q_stride_row;
} dapq_qproj;
int dapq_pseudo_queries(const dapq_qproj* desc, const void* x, const int32_t* token_idx, const void* w_q,
                        const int32_t* positions, double theta, int32_t pairing, void* q_out, void* workspace,
                        size_t workspace_bytes, void* stream);

/* Bytes of device workspace dapq_pseudo_queries needs for this description (0 for most multi-layer calls, and
 * 0 if the description is invalid: the call itself then reports why). */
size_t dapq_pseudo_queries_workspace_bytes(const dapq_qproj* desc);

/* Sec. 4.2, importance score — S(j) = sum_i Attention(q_i, k_j), summed also over the query heads
 * that share the KV head; Attention is the softmax over the L_p prompt keys of one sequence
 * (App. C.1).  Two streaming passes over K, no N x L_p matrix is stored.
 *   scores   out, fp32 [n_layers][n_kv_heads][total_tokens]
 *   workspace  device scratch of at least dapq_workspace_bytes(shape), 256-byte aligned.
 * Equivalent to dapq_score_stats followed by dapq_score_accumulate, bit for bit.  For a dense batch with at most
 * 256 query rows per KV head whose sequences split into at most 4 key chunks (dapq_score_single_launch() says
 * whether a shape is one) both passes run in one kernel: the waves of a workgroup hold one (layer, sequence, KV head),
 * merge their row statistics through LDS between the passes and keep the query fragments in registers. */
int dapq_score(const dapq_shape* shape, const void* q, const void* k, float* scores, void* workspace,
               size_t workspace_bytes, void* stream);

/* 1 if dapq_score (and dapq_score_static) runs both passes of this shape in one kernel, 0 if it runs them as
 * separate launches, a negative DAPQ_ERR_* code if the shape is invalid.  Host-only: looks at the shape and the
 * launch plan, touches no device memory. */
int dapq_score_single_launch(const dapq_shape* shape);

/* dapq_score for callers that cannot allocate device memory or hand over a workspace: code recorded into a HIP
 * graph, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same kernels and bit-identical
 * scores; the workspace of the two passes is an array of DAPQ_STATIC_SCRATCH_BYTES that the library holds in
 * device memory (one copy on every GPU it runs on, until the process ends).  The call allocates and frees
 * nothing and calls no allocating routine; its first call on a device looks up that device's copy of the array.
 *   DAPQ_ERR_WORKSPACE   dapq_workspace_bytes(shape) exceeds DAPQ_STATIC_SCRATCH_BYTES (the limit covers the
 *                        Llama-3-8B shape at L_p = 32768, N = 64, all 32 layers: 2.4 MB)
 * Every call on a GPU uses that GPU's one array, which keeps the contents of the previous call (nothing in it has
 * to be cleared: the first pass writes everything the second reads).  Two calls in flight on the same GPU at the
 * same time -- different streams, or host threads -- race on it: serialise them, or use dapq_score with
 * separate workspaces.  (A shape whose passes run in one kernel, see dapq_score_single_launch(), uses no workspace
 * at all; the size check above applies to it all the same.)  dapq_score_static_capacity() returns
 * DAPQ_STATIC_SCRATCH_BYTES as built. */
#define DAPQ_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
int dapq_score_static(const dapq_shape* shape, const void* q, const void* k, float* scores, void* stream);
size_t dapq_score_static_capacity(void);

/* First pass of dapq_score: for every pseudo query row, lse2 = log2 sum_j 2^(c*l_j) with
 * l_j = q.k_j and c = scale*log2(e), i.e. the softmax normaliser of App. C.1 Step 1 in log2 form.
 *   lse2   out, fp32 [n_layers][batch][n_q_heads][n_pseudo] */
int dapq_score_stats(const dapq_shape* shape, const void* q, const void* k, float* lse2, void* workspace,
                     size_t workspace_bytes, void* stream);

/* Second pass of dapq_score: recomputes the logits, forms alpha = 2^(c*l - lse2) and writes its
 * sum over the pseudo queries and the group for every key.  lse2 as written by dapq_score_stats
 * (it may live outside the workspace; inside it only the region dapq_score itself uses is safe). */
int dapq_score_accumulate(const dapq_shape* shape, const void* q, const void* k, const float* lse2,
                          float* scores, void* workspace, size_t workspace_bytes, void* stream);

/* Sec. 4.1 prefills the pseudo tokens in the same sequence as the prompt, so pseudo query i (position
 * L_p+i) also attends, causally, to the keys of the pseudo tokens at positions L_p..L_p+i.  This call
 * adds that block to the normaliser written by dapq_score_stats, in place:
 *   lse2[row i] <- log2( 2^lse2[row i] + sum_{t<=i} 2^(c * q_i.kp_t) ),
 * after which dapq_score_accumulate yields S(j) over the prompt keys with every softmax row
 * normalised over the extended sequence (the rows then sum to less than 1 over the prompt keys).
 *   k_pseudo   device, bf16, the pseudo tokens' own keys after RoPE: element (layer, seq, kv head,
 *              t, c) at kp_stride_layer*layer + kp_stride_seq*seq + kp_stride_head*head +
 *              kp_stride_row*t + c (strides in elements, rows of head_dim contiguous, 16-byte aligned)
 *   lse2       in/out, fp32 [n_layers][batch][n_q_heads][n_pseudo]
 * Uses q and the q strides of shape; the K/V strides and cu_seqlens are not read. */
int dapq_score_stats_extend(const dapq_shape* shape, const void* q, const void* k_pseudo,
                            int64_t kp_stride_layer, int64_t kp_stride_seq, int64_t kp_stride_head,
                            int64_t kp_stride_row, float* lse2, void* stream);

/* Pooling of the accumulated scores before selection (Sec. 1 / Sec. 5.1: selection runs on pooled
 * accumulated attention scores): pooled(j) = max of scores over |t-j| <= (width-1)/2 inside the
 * same sequence (the window is clipped at the sequence ends).  width odd, 1 <= width <= 63.
 * pooled must not alias scores. */
int dapq_pool(const dapq_shape* shape, const float* scores, float* pooled, int32_t width, void* stream);

/* Sec. 4.2, M_retain = TopK_j S(j).  For every (layer, sequence, KV head): the min(budget, L_p)
 * positions with the largest pooled score; equal scores are taken lowest position first; the
 * result is written in ascending position.  Scores must be non-negative and finite.
 *   budget           slots per head in idx (>= 1)
 *   budget_per_seq   optional device int32 [batch]: budget of each sequence (clamped to [0, budget]); NULL = budget
 *   idx, count       out; idx slots past count are left untouched
 *   workspace, workspace_bytes   optional device scratch of dapq_topk_workspace_bytes() bytes (256-byte aligned).
 *                    Heads of up to 32768 keys are selected by one workgroup each, out of its registers, and never
 *                    use it.  With the workspace, longer heads are selected in pieces of 32768 keys whose survivors
 *                    go to candidate lists in the workspace and are then selected among.  Without it (NULL or too
 *                    small) heads of up to 65536 keys still fit one workgroup (64 keys per thread, slower per key),
 *                    and longer ones are streamed from memory five times by one workgroup each: the same result,
 *                    several times slower.  Contents need not be initialised and mean nothing after the call; calls
 *                    that share a workspace must not overlap. */
int dapq_topk(const dapq_shape* shape, const float* pooled, int32_t budget, const int32_t* budget_per_seq,
              int32_t* idx, int32_t* count, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of the optional workspace of dapq_topk / dapq_pool_topk for this shape and budget: 0 if no head can have more
 * than 32768 keys (a ragged batch: more than the workgroup size chosen for its mean length), if the candidates of a
 * head would be more than 65536, or if the shape is invalid; else 2 x 4 bytes per candidate slot
 * (heads x pieces x budget) plus a count per piece.  Host arithmetic only. */
size_t dapq_topk_workspace_bytes(const dapq_shape* shape, int32_t budget);

/* dapq_pool followed by dapq_topk as one call.  For width <= 9 the selection kernels pool on the way in (each thread
 * pools its run of scores in registers, window clipped at the sequence ends) and the pooled scores never travel
 * through HBM: always when every head has at most 65536 keys, and for longer heads when the workspace of
 * dapq_topk_workspace_bytes() is passed (heads in pieces pool across the piece boundaries).  `pooled` may then be NULL,
 * and if it is not NULL it receives the pooled scores as dapq_pool would write them.  Otherwise the two kernels
 * run one after the other and `pooled` (fp32 [n_layers][n_kv_heads][total_tokens], not aliasing
 * scores) is required as the intermediate: DAPQ_ERR_UNSUPPORTED if it is NULL.  Results are identical
 * to the two separate calls in every case.  workspace, workspace_bytes: as for dapq_topk (may be NULL, 0). */
int dapq_pool_topk(const dapq_shape* shape, const float* scores, int32_t width, int32_t budget,
                   const int32_t* budget_per_seq, int32_t* idx, int32_t* count, float* pooled, void* workspace,
                   size_t workspace_bytes, void* stream);

/* Sec. 4.2 — cache pruning: copies the retained K and V rows, bit for bit, into the compact cache;
 * nothing of the pseudo segment is kept.  Rows past count are left untouched.
 * k_out / v_out must not overlap k / v. */
int dapq_gather(const dapq_shape* shape, const void* k, const void* v, const int32_t* idx,
                const int32_t* count, int32_t budget, void* k_out, void* v_out, void* stream);

/* Sec. 3.3, recall of an eviction decision: Recall_W = |M_gold ∩ M_pred| / |M_gold| for every
 * (layer, sequence, KV head).  Both index sets are in dapq_topk's format (ascending, distinct
 * positions; idx_* int32 [n_layers][batch][n_kv_heads][budget_*], count_* int32
 * [n_layers][batch][n_kv_heads]; only the first count entries of a head are read).
 *   common   out, int32 [n_layers][batch][n_kv_heads]: |M_gold ∩ M_pred|
 *   recall   out, fp32 same shape, or NULL: common / count_gold (0 where count_gold is 0) */
int dapq_recall(const dapq_shape* shape, const int32_t* idx_gold, const int32_t* count_gold, int32_t budget_gold,
                const int32_t* idx_pred, const int32_t* count_pred, int32_t budget_pred, int32_t* common,
                float* recall, void* stream);

/* Sec. 4.2, last paragraph: after pruning, decoding starts at position L_p and uses only the compressed
 * cache.  One decode step of attention over the compact cache dapq_gather wrote:
 *   out[layer][seq][h] = softmax(q K_c^T * scale) V_c   over the first count rows of KV head h / (H_q/H_kv)
 *   q_decode   device, bf16 [n_layers][batch][n_q_heads][head_dim], rotated to the decode position
 *   k_cache, v_cache   device, bf16 [n_layers][batch][n_kv_heads][budget][head_dim] (keys rotated), 16-byte aligned
 *   count      device, int32 [n_layers][batch][n_kv_heads]
 *   out        device, fp32 [n_layers][batch][n_q_heads][head_dim]; zeros where count is 0
 * budget <= 8192.  Only n_layers, batch, the head counts and scale of shape are used. */
int dapq_decode_attention(const dapq_shape* shape, const void* q_decode, const void* k_cache, const void* v_cache,
                          const int32_t* count, int32_t budget, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DAPQ_H */
