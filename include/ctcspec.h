/*
 * ctcspec.h - C ABI of libctcspec: the per-step device work of CTC-drafted speculative decoding
 * (draft head -> CTC transform -> tree verification attention -> greedy acceptance) on one AMD
 * MI355X (gfx950).
 *
 * Conventions that hold for every call
 *  - Plain C.  Every data pointer is a DEVICE pointer owned by the caller unless a comment says
 *    "host".  The library never allocates, frees or keeps caller buffers; it owns only the
 *    workspace that ctcspec_create allocates inside the context.
 *  - All work is enqueued on the HIP stream given to ctcspec_create / ctcspec_set_stream.  No call
 *    synchronises with the host.  Sizes that depend on the data (n_cand, n_nodes) are written to
 *    device memory and read from there by the later calls, so the four stage calls can be issued
 *    back to back.
 *  - Return value: CTCSPEC_OK (0) or a negative error code.  On error nothing has been launched and
 *    ctcspec_last_error(ctx) describes the reason.  No C++ exception crosses this boundary.
 *  - One context serves one stream at a time: calls on the same context from several threads, or
 *    overlapping on the GPU, race on its workspace.
 *  - Row-major, innermost index last, no padding unless stated.  bf16 is the upper half of an IEEE
 *    float32 (1-8-7).  int32_t/int64_t/uint64_t are little endian device integers.
 *
 * Notation: B sequences, T draft slots, D hidden size, V vocabulary size (the blank is one extra
 * row, id V, so the head has V+1 rows), k tokens kept per slot, H heads, dh head dimension.
 */
#ifndef CTCSPEC_H
#define CTCSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ctcspec_ctx ctcspec_ctx;

typedef enum { CTCSPEC_F32 = 0, CTCSPEC_BF16 = 1 } ctcspec_dtype;

enum {
  CTCSPEC_OK = 0,
  CTCSPEC_EINVAL = -1,       /* null / misaligned pointer, non-positive size, inconsistent arguments */
  CTCSPEC_EUNSUPPORTED = -2, /* shape outside the compiled limits or the context's limits */
  CTCSPEC_EHIP = -3          /* the HIP runtime reported a failure */
};

/* Compiled limits. */
#define CTCSPEC_MAX_SLOTS 8        /* T */
#define CTCSPEC_MAX_TOPK 8         /* k */
#define CTCSPEC_MAX_ALIGNMENTS 65536 /* k^T */
#define CTCSPEC_MAX_BEAM 128
#define CTCSPEC_MAX_NODES 128      /* tree nodes per sequence, root included */
#define CTCSPEC_MAX_COLUMNS 64     /* B*T columns of one draft-head call */
#define CTCSPEC_MAX_HEAD_DIM 128
#define CTCSPEC_NOALLOC_MAX_VOCAB_ROWS 65536 /* V+1 of ctc_draft_topk_noalloc */

/* Sizes the context's workspace is dimensioned for.  Calls that exceed them fail with
 * CTCSPEC_EUNSUPPORTED. */
typedef struct {
  int max_batch;      /* B */
  int max_slots;      /* T  <= CTCSPEC_MAX_SLOTS */
  int max_topk;       /* k  <= CTCSPEC_MAX_TOPK */
  int max_vocab_rows; /* V+1 */
  int max_nodes;      /* <= CTCSPEC_MAX_NODES */
  int max_heads;      /* H */
  int max_head_dim;   /* dh <= CTCSPEC_MAX_HEAD_DIM */
} ctcspec_limits;

/* Create a context: allocates the device workspace on the current HIP device (this is the only
 * place the library allocates device memory) and binds `hip_stream` (a hipStream_t; NULL = the
 * default stream).  *out is set to NULL on failure.  Host pointers. */
int ctcspec_create(ctcspec_ctx** out, void* hip_stream, const ctcspec_limits* limits);

/* Free the workspace.  The caller must have synchronised the stream.  NULL is ignored. */
void ctcspec_destroy(ctcspec_ctx* ctx);

/* Bind another stream for subsequent calls (work already enqueued stays where it is). */
int ctcspec_set_stream(ctcspec_ctx* ctx, void* hip_stream);

/* Static, NUL-terminated description of the last error on this context ("" if none).  With
 * ctx == NULL: the reason the last call without a context (ctcspec_create, ctc_draft_topk_noalloc) failed in this
 * thread. */
const char* ctcspec_last_error(const ctcspec_ctx* ctx);

/* Bytes of device workspace the context holds. */
size_t ctcspec_workspace_bytes(const ctcspec_ctx* ctx);

/* Deferred merge of the draft head.  ctc_draft_topk runs one pass over the head weights that leaves a partial
 * result per 128 vocabulary rows, and a small second kernel that merges them into topk_id / topk_logp / lse.  With
 * enable != 0 that second kernel is not launched: the three outputs stay OWED until the next call on this context -
 *   - ctc_collapse_tree given exactly those topk_id / topk_logp buffers (same B*T, k <= 4) merges the partials in the
 *     prologue of its own kernel and writes the three outputs as well: one dispatch and one trip through memory
 *     fewer per decoding step, same bits;
 *   - any other library call on the context, ctcspec_set_stream and ctcspec_flush launch the merge kernel first.
 * A caller that reads the three outputs from the stream with code of its own right after ctc_draft_topk must call
 * ctcspec_flush first, or leave the mode off (the default).  ctcspec_destroy drops an unsettled debt. */
int ctcspec_defer_topk_merge(ctcspec_ctx* ctx, int enable);
int ctcspec_flush(ctcspec_ctx* ctx);

/* Measurement aid.  With enable != 0, every following ctc_draft_topk call attaches a pair of HIP events
 * to the launch of its main kernel on the context's stream (the pass over the head weights, not the
 * small merge kernel): the events take that kernel's begin and end timestamps.  (The many-column and
 * generic producers record the pair around the launch instead, which also spans the dispatch.)
 * ctcspec_draft_head_kernel_ms synchronises with the second event of the LAST
 * such call and returns the elapsed milliseconds in *ms (host pointer).  CTCSPEC_EINVAL when profiling
 * is off or no call has been made since it was switched on. */
int ctcspec_profile_draft_head(ctcspec_ctx* ctx, int enable);
int ctcspec_draft_head_kernel_ms(ctcspec_ctx* ctx, float* ms);

/* Measurement aid.  Reads the first floor(bytes / 131072) * 131072 bytes at src (device, 16-byte aligned) once, with
 * coalesced 16-byte loads and nothing else, on the context's stream: the rate this GPU delivers to a kernel that
 * streams a matrix, against which the HBM-bound kernels' rates can be set beside the nominal peak.  sink: one device
 * word that is (practically) never written.  Timing is the caller's (events on the stream). */
int ctcspec_stream_probe(ctcspec_ctx* ctx, const void* src, size_t bytes, uint32_t* sink);

/*
 * Stage 1+2 - draft head.  For every draft slot, project its hidden state through the LM head of
 * the augmented vocabulary (tokens plus blank), take the log-softmax over all V+1 entries and keep
 * the k most probable entries in descending order (paper Sec. 3.2: P^ = Softmax(LmHead(F^)), the
 * blank being one more output symbol, Sec. 2.2; Sec. 3.3: "for every position the top k tokens").
 *
 *   z[b,t,v]   = sum_d hidden[b,t,d] * w[v,d] + bias[v]       (fp32 accumulate)
 *   lse[b,t]   = log sum_v exp z[b,t,v]
 *   topk_id    = the k indices of largest z[b,t,:], descending; equal z -> smaller index first
 *   topk_logp  = z[topk_id] - lse
 *
 * dt           element type of hidden and w (CTCSPEC_F32: float, CTCSPEC_BF16: bf16)
 * hidden       [B,T,D]            16-byte aligned
 * w            [Vp1,D] row-major  16-byte aligned; row Vp1-1 is the blank unless the caller decides
 *                                 otherwise (this call does not treat any row specially)
 * bias         [Vp1] float or NULL (= 0)
 * topk_id      [B,T,k] int32   out
 * topk_logp    [B,T,k] float   out
 * lse          [B,T]   float   out, may be NULL
 * logits_out   [B,T,Vp1] float out, may be NULL; when given, receives exactly the z values the
 *              ranking used (for parity checks; costs extra HBM writes)
 * Limits: B*T <= CTCSPEC_MAX_COLUMNS, 1 <= k <= min(CTCSPEC_MAX_TOPK, Vp1), Vp1 <= limits.
 */
int ctc_draft_topk(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* hidden, const void* w,
                   const float* bias, int B, int T, int D, int Vp1, int k, int32_t* topk_id,
                   float* topk_logp, float* lse, float* logits_out);

/*
 * ctc_draft_topk_noalloc - ctc_draft_topk for callers that cannot allocate device memory and therefore cannot create
 * a context: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation,
 * same kernels, same outputs bit for bit; it takes the stream instead of a context and keeps its partial results
 * (per 128 vocabulary rows and column: max, sum of exponentials, k best keys) in a device array that is part of the
 * library's own code object, so that no call of it, first or later, allocates or frees anything (neither through
 * HIP nor through any other library).
 *
 * hip_stream   a hipStream_t (NULL = the default stream); host value
 * every other argument as for ctc_draft_topk
 * Limits: Vp1 <= CTCSPEC_NOALLOC_MAX_VOCAB_ROWS (larger heads are rejected with CTCSPEC_EUNSUPPORTED: use a context),
 * B*T <= CTCSPEC_MAX_COLUMNS, k <= CTCSPEC_MAX_TOPK, T <= CTCSPEC_MAX_SLOTS.  The array (2.4 MB) exists once per GPU
 * for the life of the process, and every call on a GPU uses it: calls that overlap on one GPU (two streams, two
 * threads) race on it; calls in stream order are safe and need no clearing between them (every entry a call reads
 * it has written first).  Errors are reported through ctcspec_last_error(NULL).
 */
int ctc_draft_topk_noalloc(void* hip_stream, ctcspec_dtype dt, const void* hidden, const void* w,
                           const float* bias, int B, int T, int D, int Vp1, int k, int32_t* topk_id,
                           float* topk_logp, float* lse, float* logits_out);

/*
 * Stage 3 - CTC transform and token tree (paper Sec. 3.1 "CTC Transform Module", Sec. 3.3; collapse
 * rule beta^-1 of Sec. 2.2; candidate value = Eq. 6; tree verification layout of Sec. 2.1).
 *
 * Every rank tuple r in {0..k-1}^T is a raw candidate a_t = topk_id[t, r_t] with index
 * idx(r) = sum_t r_t * k^(T-1-t) and score s(r) = (((l_0 + l_1) + l_2) + ...), l_t =
 * topk_logp[t, r_t], summed in float32 in that order.  Raw candidates are collapsed (merge adjacent
 * equal symbols, then delete blank_id); equal collapsed sequences are one draft whose score is its
 * best raw candidate's and whose representative is the best-scoring raw candidate of smallest idx;
 * the empty draft is dropped.  Drafts ordered by (score descending, representative idx ascending);
 * the first `beam` are kept.  They are inserted in that order into a prefix tree below node 0 (the
 * root, token root_token[b]): node ids are creation order, nothing is created once the tree holds
 * max_nodes nodes (drafts cut short keep their created prefix).
 *
 * topk_id, topk_logp  [B,T,k]   in (as written by ctc_draft_topk; logp descending per slot is
 *                     not required)
 * root_token   [B] int32        in: the base model's own greedy token
 * n_cand       [B] int32        out: drafts kept (<= beam)
 * cand_tokens  [B,beam,T] int32 out, unused positions -1
 * cand_len     [B,beam] int32   out, 0 beyond n_cand
 * cand_score   [B,beam] float   out, -inf beyond n_cand
 * cand_leaf    [B,beam] int32   out: node of the draft's last token, -1 if cut by the node cap or
 *                               beyond n_cand
 * n_nodes      [B] int32        out: 1..max_nodes
 * node_token, node_parent, node_depth  [B,max_nodes] int32 out; root: parent -1, depth 0; entries
 *                               beyond n_nodes are -1
 * anc_mask     [B,max_nodes,ceil(max_nodes/64)] uint64 out: bit (j%64) of word j/64 of row i is 1
 *              iff node j is on the path root..i (both ends included); rows beyond n_nodes are 0
 * Limits: T <= CTCSPEC_MAX_SLOTS, k <= CTCSPEC_MAX_TOPK, k^T <= CTCSPEC_MAX_ALIGNMENTS,
 * 1 <= beam <= CTCSPEC_MAX_BEAM, 1 <= max_nodes <= CTCSPEC_MAX_NODES.
 */
int ctc_collapse_tree(ctcspec_ctx* ctx, const int32_t* topk_id, const float* topk_logp,
                      const int32_t* root_token, int B, int T, int k, int32_t blank_id, int beam,
                      int max_nodes, int32_t* n_cand, int32_t* cand_tokens, int32_t* cand_len,
                      float* cand_score, int32_t* cand_leaf, int32_t* n_nodes, int32_t* node_token,
                      int32_t* node_parent, int32_t* node_depth, uint64_t* anc_mask);

/*
 * Stage 4a - one attention layer of the base model's parallel verification pass over the token tree
 * (paper Sec. 2.1 tree verification, Sec. 3.1 masked attention map, Sec. 3.3 "all candidates are
 * verified parallelly").  For sequence b, head h and node i < n_nodes[b]:
 *
 *   keys(i) = the ctx_len[b] cached positions (all visible) + the tree nodes j with bit j of
 *             anc_mask row i set
 *   out[b,h,i,:] = sum_{j in keys(i)} softmax_j(scale * q[b,h,i,:] . key_j) * value_j
 *
 * No positional encoding is applied here: q and keys arrive as the attention operands.
 *
 * dt           element type of q, k_cache, v_cache, k_tree, v_tree
 * q, k_tree, v_tree   [B,H,max_nodes,dh]   16-byte aligned; rows >= n_nodes[b] are never used
 * k_cache, v_cache    base pointers; sequence b's block starts kv_off[b] ELEMENTS after the base and
 *                     is laid out [H][kv_cap][dh]; only the first ctx_len[b] rows of each head are
 *                     read (rows beyond may hold anything, NaN included).  kv_off[b]*sizeof(elem)
 *                     must be a multiple of 16.
 * kv_off       [B] int64 device, ctx_len [B] int32 device (0 <= ctx_len[b] <= kv_cap)
 * n_nodes      [B] int32 device, anc_mask as written by ctc_collapse_tree
 * scale        softmax scale, normally 1/sqrt(dh)
 * out          [B,H,max_nodes,dh] float out; rows >= n_nodes[b] are unspecified
 * Limits: dh <= CTCSPEC_MAX_HEAD_DIM and dh % 8 == 0, max_nodes <= CTCSPEC_MAX_NODES, H <= limits.
 */
int tree_verify_attn(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* q, const void* k_cache,
                     const void* v_cache, const int64_t* kv_off, const int32_t* ctx_len, int kv_cap,
                     const void* k_tree, const void* v_tree, const int32_t* n_nodes,
                     const uint64_t* anc_mask, int B, int H, int dh, int max_nodes, float scale,
                     float* out);

/*
 * Stage 4b - greedy acceptance (paper Sec. 2.1: accept what matches the target model's greedy
 * output; Sec. 3.3: "the longest sequence that satisfies the criterion").  target_argmax[b,i] is
 * the base model's greedy token after node i.  From the root, step to the child whose token equals
 * target_argmax at the current node; stop when there is none.
 *
 * n_nodes, node_token, node_parent, node_depth   as written by ctc_collapse_tree
 * target_argmax [B,max_nodes] int32 in
 * accept_len    [B] int32 out: draft tokens accepted (0..T); the root is always part of the output
 * accept_nodes  [B,T+1] int32 out: the accepted path, root first, -1 beyond
 * accept_tokens [B,T+1] int32 out: tokens of those nodes, -1 beyond
 * next_token    [B] int32 out: target_argmax at the last accepted node (the bonus token)
 */
int accept_longest(ctcspec_ctx* ctx, const int32_t* n_nodes, const int32_t* node_token,
                   const int32_t* node_parent, const int32_t* node_depth,
                   const int32_t* target_argmax, int B, int T, int max_nodes, int32_t* accept_len,
                   int32_t* accept_nodes, int32_t* accept_tokens, int32_t* next_token);

/*
 * Closing the step, part 1 - the base model's greedy token after every tree node (paper Sec. 3.1: the
 * base model ends in an LM head that maps hidden states to the vocabulary; Sec. 2.1 / 3.3: candidates
 * are verified against the base model's greedy output).  For sequence b and node i < n_nodes[b]:
 *
 *   z[v] = sum_d node_hidden[b,i,d] * w_base[v,d]          (fp32 accumulation)
 *   target_argmax[b,i] = argmax_v z[v], the smaller id among equal logits
 *
 * This produces the target_argmax input of accept_longest; rows i >= n_nodes[b] receive -1.
 *
 * dt            element type of node_hidden and w_base
 * node_hidden   [B,max_nodes,D]    16-byte aligned: the base model's last hidden state at every tree node
 *               (rows >= n_nodes[b] are read and must be readable; their results are discarded)
 * w_base        [V,D] row-major    16-byte aligned: the base model's LM head (no blank row)
 * n_nodes       [B] int32 device
 * target_argmax [B,max_nodes] int32 out
 * logits_out    [B,max_nodes,V] float out, may be NULL; when given, receives exactly the z values the
 *               argmax used (for parity checks; costs extra HBM writes)
 * One pass over the weights in HBM whatever the number of nodes: blocks of 128 node columns that share a block of
 * weight rows are scheduled next to each other on one XCD, so that all but the first find the rows in its L2.
 * Limits: B, max_nodes, V within the context's limits (V <= max_vocab_rows).
 */
int verify_head_argmax(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* node_hidden, const void* w_base,
                       const int32_t* n_nodes, int B, int max_nodes, int D, int V,
                       int32_t* target_argmax, float* logits_out);

/*
 * Closing the step, part 2 - history update (paper Sec. 3.3: "the decoding history is updated according
 * to the output").  The keys and values of the accepted path - the root, which is the base model's own
 * token, then the accept_len[b] accepted draft tokens, in path order - are appended to sequence b's cached
 * context in one attention layer:
 *
 *   for j = 0..accept_len[b]:  cache row ctx_len[b] + j of every head  <-  tree row accept_nodes[b,j]
 *   ctx_len_out[b] = min(ctx_len[b] + accept_len[b] + 1, kv_cap)
 *
 * Rows that would fall beyond kv_cap are dropped, and ctx_len_out counts only the rows the cache then holds: a
 * sequence lost accepted rows exactly when ctx_len_out[b] < ctx_len[b] + accept_len[b] + 1 (the caller sizes
 * kv_cap so that this cannot happen, or checks that relation before the next step).  One call per layer; layers
 * share accept_* and ctx_len, so pass ctx_len_out only with the last layer (NULL otherwise).  Buffers of any
 * alignment are accepted; 16-byte aligned ones (pointers, kv_off and row size) are copied 16 bytes at a time.
 *
 * dt            element type of the K/V buffers
 * k_tree, v_tree  [B,H,max_nodes,dh]  in (as given to tree_verify_attn)
 * accept_len    [B] int32, accept_nodes [B,T+1] int32   as written by accept_longest
 * kv_off, ctx_len, kv_cap, k_cache, v_cache   as for tree_verify_attn; the caches are written
 * ctx_len_out   [B] int32 out or NULL; must not be the ctx_len buffer itself
 */
int kv_commit(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* k_tree, const void* v_tree,
              const int32_t* accept_len, const int32_t* accept_nodes, int T, const int64_t* kv_off,
              const int32_t* ctx_len, int kv_cap, int B, int H, int dh, int max_nodes, void* k_cache,
              void* v_cache, int32_t* ctx_len_out);

/*
 * draft_layer_forward - the transformer layer of the attention draft module (Sec. 3.1 "Model Structure": one
 * transformer layer of the base model's construction over the base model's last hidden states, predicting all
 * draft positions in parallel; its output goes to the LM head, i.e. to ctc_draft_topk).
 *
 * The layer is the base family's decoder layer (Vicuna/LLaMA), for column (b, t), t = 0..T-1, at position
 * pos0[b] + t:
 *   h   = RMSNorm(x; ln1)                      y / sqrt(mean(y^2) + rms_eps) * gain
 *   q, k, v = h Wq^T, h Wk^T, h Wv^T           head i owns output rows i*dh .. i*dh+dh-1, dh = D / H
 *   q, k <- rotary embedding                   pair (j, j + dh/2) turned by (pos0[b] + t) * rope_theta^(-2j/dh)
 *   a   = softmax(q K^T / sqrt(dh)) V          over the ctx_len[b] cached positions and the new positions <= t
 *   h1  = x + a Wo^T
 *   out = h1 + (silu(m Wg^T) * (m Wu^T)) Wd^T  with m = RMSNorm(h1; ln2)
 * The cache is read only; k_new (rotated) and v_new are returned so that the caller appends what it keeps
 * (kv_commit takes them as k_tree / v_tree with max_nodes = T).
 *
 * All pointers are device pointers, 16-byte aligned, bf16 (dt must be CTCSPEC_BF16) unless stated:
 * x         [B,T,D] in
 * w         host struct of device pointers: ln1 [D], wqkv [3D,D] (rows: Wq, then Wk, then Wv), wo [D,D],
 *           ln2 [D], wgu [2F,D] (rows: Wg, then Wu), wd [D,F]; row-major, row = output feature
 * pos0      [B] int32 in
 * k_cache, v_cache, kv_off [B] int64, ctx_len [B] int32, kv_cap: the layer's cache, laid out as for
 *           tree_verify_attn ([H, kv_cap, dh] per sequence at element offset kv_off[b]); not modified
 * workspace device scratch of at least draft_layer_workspace_bytes(B, T, D, H, F) bytes, owned by the
 *           caller, contents undefined afterwards; calls that share it must not overlap
 * q_out     [B,H,T,dh] out or NULL: the rotated queries the attention step used (otherwise kept in the workspace)
 * k_new, v_new [B,H,T,dh] out
 * out       [B,T,D] out;  out_f32 [B,T,D] float out or NULL: the same values before rounding to bf16
 * Limits: D % 256 == 0, F % 256 == 0, dh % 8 == 0, dh <= CTCSPEC_MAX_HEAD_DIM, T <= 64 and T <= limits.max_nodes,
 * B, H, dh within the context's limits.  Returns CTCSPEC_OK or an error code (see ctcspec_last_error);
 * nothing is written on an argument error.  Work is queued on the context's stream.
 */
typedef struct {
  const void* ln1;
  const void* wqkv;
  const void* wo;
  const void* ln2;
  const void* wgu;
  const void* wd;
} ctcspec_layer_weights;

size_t draft_layer_workspace_bytes(int B, int T, int D, int H, int F);

int draft_layer_forward(ctcspec_ctx* ctx, ctcspec_dtype dt, const void* x, const ctcspec_layer_weights* w,
                        const int32_t* pos0, void* k_cache, void* v_cache, const int64_t* kv_off,
                        const int32_t* ctx_len, int kv_cap, int B, int T, int D, int H, int F, float rms_eps,
                        float rope_theta, void* workspace, size_t workspace_bytes, void* q_out, void* k_new,
                        void* v_new, void* out, float* out_f32);

/*
 * ctc_sum_score - value of the candidate drafts under Eq. 5 (Sec. 3.2): log P(Y|X) summed over every raw
 * sequence of T tokens, from the whole vocabulary plus the blank, that the collapse rule turns into Y, each
 * raw sequence weighted by Eq. 6; computed with the forward recursion of the CTC paper the section cites.
 * ctc_collapse_tree values a draft by its best alignment alone; this is the alternative, and the rank order it
 * induces.  Takes the optional logits output and the lse output of ctc_draft_topk and the candidate lists of
 * ctc_collapse_tree; changes neither.
 *
 * logits        [B,T,Vp1] float device in
 * lse           [B,T] float device in: log p_t(v) = logits[b,t,v] - lse[b,t]
 * cand_tokens   [B,beam,T] int32 device in; cand_len [B,beam] int32 device in; n_cand [B] int32 device in
 * cand_logp_sum [B,beam] float device out, -inf beyond n_cand (and for a draft longer than T slots can hold)
 * cand_rank_sum [B,beam] int32 device out: position of candidate i in the order (cand_logp_sum descending,
 *               index ascending), decided on the fp32 values; -1 beyond n_cand
 * Limits: T <= CTCSPEC_MAX_SLOTS, beam <= CTCSPEC_MAX_BEAM, B within the context's limits.
 */
int ctc_sum_score(ctcspec_ctx* ctx, const float* logits, const float* lse, const int32_t* cand_tokens,
                  const int32_t* cand_len, const int32_t* n_cand, int B, int T, int Vp1, int32_t blank_id, int beam,
                  float* cand_logp_sum, int32_t* cand_rank_sum);

/*
 * ctc_raw_tree - the tree layout that Sec. 3.1 describes literally, as an alternative to ctc_collapse_tree: the
 * raw candidates keep their full length T (blanks and repeats included) and form the token tree as they are; the
 * CTC transform marks the positions it removes (a blank; a token equal to the raw token of the slot before it -
 * the root is no slot) and the attention map hides those positions from everything below them.
 * Same arguments, layouts, limits and error behaviour as ctc_collapse_tree, with these differences:
 * candidates   the `beam` best raw candidates (Eq. 6 value, ties to the smaller index), not collapsed:
 *              cand_tokens holds raw tokens (the blank id included), cand_len = T
 * tree         prefix tree over raw tokens, same node cap rule
 * anc_mask     bit j of row i: j == i, or j an ancestor of i (the root included) that is not removed
 * node_removed [B,max_nodes] int32 device out: 1 removed, 0 kept, -1 beyond n_nodes
 * tree_verify_attn takes the result unchanged; a kept node's output equals that of the collapsed tree's node for
 * the same collapsed prefix.  The layout spends nodes on removed positions: under the same node cap it holds
 * fewer distinct drafts, which is why the step uses ctc_collapse_tree.
 */
int ctc_raw_tree(ctcspec_ctx* ctx, const int32_t* topk_id, const float* topk_logp, const int32_t* root_token, int B,
                 int T, int k, int32_t blank_id, int beam, int max_nodes, int32_t* n_cand, int32_t* cand_tokens,
                 int32_t* cand_len, float* cand_score, int32_t* cand_leaf, int32_t* n_nodes, int32_t* node_token,
                 int32_t* node_parent, int32_t* node_depth, uint64_t* anc_mask, int32_t* node_removed);

/*
 * verify_sample_tokens - sampling-based acceptance (Sec. 2.1: a drafted token is accepted with probability
 * min(1, P/P') and a rejected one re-drawn from norm(max(0, P - P')); Sec. 3.3: the longest sequence that satisfies
 * the criterion is the step's output).  The tree is built deterministically, so the draft distribution behind a
 * node's token is a point mass; the rule then emits tokens with the target model's own distribution, which one
 * uniform number per node realises: draw the target's token after the node; accept_longest, given these tokens in
 * place of the greedy ones, walks to the child that carries the drawn token and stops where none does.
 * For sequence b and node i < n_nodes[b]:
 *
 *   p[v] = softmax_v(logits[b,i,:] / temperature)
 *   target_sampled[b,i] = the first v, in vocabulary order, with p[0] + ... + p[v] > uniforms[b,i]
 *
 * (the last v with p[v] > 0 when rounding leaves no such v).  Sums are fp32 in a fixed order: the token is the exact
 * one unless uniforms[b,i] lies within rounding (about 1e-6) of a boundary of the cumulative distribution, where
 * it may be the neighbour.  Rows i >= n_nodes[b] receive -1.
 *
 * logits         [B,max_nodes,V] float device in, 16-byte aligned: the target model's logits after every node (the
 *                logits_out of verify_head_argmax)
 * n_nodes        [B] int32 device in
 * uniforms       [B,max_nodes] float device in: independent uniform numbers in [0, 1), drawn by the caller
 * temperature    > 0, finite
 * target_sampled [B,max_nodes] int32 device out
 * Limits: V <= 65533, B <= 65535.  The same bits on every run.
 */
int verify_sample_tokens(ctcspec_ctx* ctx, const float* logits, const int32_t* n_nodes, const float* uniforms,
                         float temperature, int B, int max_nodes, int V, int32_t* target_sampled);

/*
 * ctc_loss - the training objective of Sec. 3.2: for every sequence b the loss -log P(Y_b | X_b), P by Eq. 5 with
 * Eq. 6 (the sum, over all frame-level sequences that the collapse rule turns into the label, of the product of
 * the per-frame softmax probabilities), and optionally its gradient with respect to the logits - computed with
 * the forward-backward recursions of the CTC paper the section cites.  The softmax over the V+1 entries of a frame
 * is part of the differentiated function.
 *
 * logits     [B,T,Vp1] float device in: the draft module's outputs for T frames per sequence
 * labels     [B,Lmax] int32 device in: label tokens in [0, Vp1) other than blank_id, padded; label_len [B] int32
 *            device in.  Ids outside the range are clamped into it and a blank among the labels gets no
 *            gradient of its own: the values are then unspecified, nothing is read or written out of bounds
 * frame_len  [B] int32 device in: frames of sequence b that count (<= T)
 * workspace  device scratch of at least ctc_loss_workspace_bytes(B, T, Lmax) bytes, owned by the caller, contents
 *            undefined afterwards; calls that share it must not overlap
 * loss       [B] float device out; +inf when the label cannot be reached in frame_len frames
 * grad       [B,T,Vp1] float device out or NULL: d loss[b] / d logits[b,t,v]; zero for frames past frame_len and
 *            for sequences whose loss is +inf
 * Limits: Lmax <= 2047, Vp1 <= 65536, B <= 65535; logits and grad 16-byte aligned.  The same bits on every run.
 */
size_t ctc_loss_workspace_bytes(int B, int T, int Lmax);

int ctc_loss(ctcspec_ctx* ctx, const float* logits, const int32_t* labels, const int32_t* label_len,
             const int32_t* frame_len, int B, int T, int Vp1, int Lmax, int32_t blank_id, void* workspace,
             size_t workspace_bytes, float* loss, float* grad);

#ifdef __cplusplus
}
#endif
#endif /* CTCSPEC_H */
