/*
 * specpv.h -- C ABI of the SpecPV verification-attention library for MI355X (gfx950).
 *
 * The library implements the verification hot path of SpecPV ("partial
 * verification" self-speculative decoding for long contexts): per-block key
 * summaries (Section 3.2, eq. 1), query-aware block scores (eq. 2, eq. 3),
 * selection of sink + top-k retrieval + local blocks (Section 3.2), tree-masked
 * grouped-query attention of the draft tree over only the selected blocks
 * (Section 3.2; tree decode of Algorithm 1), and the periodic full-verification
 * pass that attends over the whole cache and refreshes the selection
 * (Section 3.3).
 *
 * Conventions for every entry point
 *  - extern "C"; returns SPECPV_OK (0) or a negative specpv_status; never throws.
 *  - Pointers inside the descriptor structs and all buffer arguments are DEVICE
 *    pointers owned by the caller, except where "host" is stated.  The structs
 *    themselves are HOST memory and are only read during the call.
 *  - No allocation and no host synchronisation happen inside a call: kernels are
 *    enqueued on `stream` (a hipStream_t passed as void*; NULL = null stream) and
 *    outputs are valid once the stream reaches that point.
 *  - Arguments are validated on the host before anything is launched; on error
 *    nothing has been enqueued.  Device-side quantities (ctx_len, sel_count,
 *    entries of sel_idx, parent) are bounds-checked inside the kernels: blocks or
 *    tokens outside the sequence are ignored, they are never dereferenced.
 *  - The calls may be issued from several threads, on different streams and on different
 *    devices (the device that is current at the call is used).  The only state the library
 *    keeps is a per-device record of one-time kernel attribute set-up, guarded for concurrent
 *    first calls.  Two calls that share a workspace must be ordered by the caller (same
 *    stream, or events).
 *
 * Notation: L_b committed tokens of sequence b, B block size, nb_b = ceil(L_b/B),
 * Hq query heads, Hkv KV heads, G = Hq/Hkv, D head dim, M draft-tree nodes (the
 * query tokens of this verify step).  Query head h reads KV head h / G.
 *
 * Supported: D in {64, 128}; dtype f32 or bf16 (q, k, v, kd, vd, summaries and
 * out share one dtype); 1 <= M <= 128; 1 <= G <= 16; B >= 1; batch >= 1.
 */
#ifndef SPECPV_H
#define SPECPV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPECPV_OK = 0,
    SPECPV_EINVAL = -1,     /* null pointer, bad shape, unsupported dtype / D / strides  */
    SPECPV_EWORKSPACE = -2, /* workspace pointer null or workspace_bytes too small        */
    SPECPV_ELIMIT = -3,     /* M, G, k or block counts beyond the documented limits       */
    SPECPV_EHIP = -4        /* a HIP launch failed; see specpv_last_hip_error()           */
} specpv_status;

typedef enum { SPECPV_F32 = 0, SPECPV_BF16 = 1 } specpv_dtype;

/* eq. 3: how the per-query scores of a block are reduced to one score. */
typedef enum { SPECPV_REDUCE_MEAN = 0, SPECPV_REDUCE_MAX = 1, SPECPV_REDUCE_LAST = 2 } specpv_reduce;

/* The per-query score of a block.  SPECPV_SCORE_EQ2 is the paper's (Section 3.2, eq. 2):
 * max(q . Kmax, q . Kmin), two full inner products.  SPECPV_SCORE_CHANNEL_BOUND is the
 * per-channel form of the query-aware page selection that the section names as the
 * inspiration of its summaries: sum over the channels d of max(q[d] * Kmax[d], q[d] * Kmin[d]),
 * an upper bound of q . k for every token of the block; it is here for comparison. */
typedef enum { SPECPV_SCORE_EQ2 = 0, SPECPV_SCORE_CHANNEL_BOUND = 1 } specpv_score;

#define SPECPV_MAX_M 128
#define SPECPV_MAX_G 16

/* One layer's committed KV cache for a batch of sequences, read in place.
 * Element (b, t, g, d) of k (and v) lives at  base + b*stride_b + g*stride_h +
 * t*stride_t + d  (strides in ELEMENTS; d is contiguous; every row start must be
 * 16-byte aligned).  Both the head-major [batch, Hkv, T, D] and the token-major
 * [batch, T, Hkv, D] layouts fit.  Rows t >= ctx_len[b] are never read. */
typedef struct specpv_kv {
    const void *k, *v;
    int64_t stride_b, stride_h, stride_t;
    const int32_t *ctx_len; /* device, [batch]: L_b                                      */
    int32_t batch, n_kv_heads, head_dim, block_size;
    int32_t max_blocks;     /* >= max_b nb_b; second-to-last extent of the summary / score arrays */
    specpv_dtype dtype;
} specpv_kv;

/* The draft tree: the query tokens of this verify step, and their own K/V (the
 * "buffer" part of the partial cache, Section 3.2).  The partially verified
 * tokens are a chain prefix of parent[] (Section 3.3): on a refresh step they are
 * verified again, i.e. they are ordinary nodes; on a partial step they are only
 * attended, i.e. the first n_key_only nodes have K/V rows and parent entries but
 * NO query rows and no output rows.  Mq = M - n_key_only is the number of query
 * nodes; query row r belongs to node n_key_only + r.
 * The key-only nodes must be that chain (parent[i] = i - 1 for 0 < i < n_key_only) and every
 * query node must descend from its last node, as specpv_extend_parents builds it: every query
 * row then attends every key-only node, and the bf16 kernels take those K/V rows along with the
 * cache tokens without looking at their parent entries (a tree that breaks the rule is not
 * detected: its query rows attend all key-only nodes all the same). */
typedef struct specpv_tree {
    const void *q;         /* [batch, Mq, Hq, D] contiguous, post-RoPE                   */
    const void *kd, *vd;   /* [batch, M, Hkv, D] contiguous; may be NULL for select      */
    const int32_t *parent; /* device, [batch, M]; parent[0] = -1, parent[i] < i          */
    int32_t M, n_q_heads;
    int32_t last_node;     /* node whose queries SPECPV_REDUCE_LAST keeps (normally the
                              tree root: n_key_only); n_key_only <= last_node < M        */
    int32_t n_key_only;    /* 0 <= n_key_only < M                                        */
} specpv_tree;

/* Composition of the partial cache in blocks (Section 3.2): always the first
 * n_sink_blocks, always the last n_recent_blocks, and the k_blocks best-scoring
 * blocks in between. */
typedef struct specpv_select_cfg {
    int32_t n_sink_blocks, n_recent_blocks, k_blocks;
    specpv_reduce reduce;
    specpv_score score;    /* SPECPV_SCORE_EQ2 (= 0) is the paper's                        */
    int32_t n_extra_slots; /* free entries behind the ns + k + nr of a list row, for the blocks
                              that later commits append (specpv_commit_accepted); >= 0       */
} specpv_select_cfg;

/* Bytes of workspace that any of the calls below needs for these descriptors
 * (host-only computation; 0 on invalid descriptors).  cfg may be NULL if only
 * specpv_block_summarize is used.
 * A workspace must be ZERO-FILLED ONCE before its first use (hipMemset, torch.zeros): its first
 * 64 KiB hold the arrival words through which the workgroups of the single-kernel route of
 * specpv_partial_verify_attn (specpv_debug_set_route) find out which of them finishes a row tile, and
 * those of the one-launch route of the selection (specpv_debug_set_select_route) which of them selects.
 * Every call leaves them zero again, so one fill at
 * allocation is enough, whatever shapes use the workspace afterwards.  A call that is given
 * words that are not zero computes garbage (it cannot notice). */
size_t specpv_workspace_bytes(const specpv_kv *kv, const specpv_tree *tree, const specpv_select_cfg *cfg);

/* Section 3.2, eq. 1.  For every sequence b, KV head g and block i in
 * [blk_begin, blk_end) (blk_end < 0: up to nb_b; blocks >= nb_b are skipped):
 *   kmax[b, g, i, :] = element-wise max of k over the block's tokens t < L_b,
 *   kmin likewise.  kmax / kmin: [batch, Hkv, max_blocks, D], kv dtype.
 * Exact in any dtype (only comparisons). */
int specpv_block_summarize(const specpv_kv *kv, int32_t blk_begin, int32_t blk_end,
                           void *kmax, void *kmin, void *stream);

/* Section 3.2, eq. 2 + eq. 3 + block selection.  Per (b, g):
 *   s[i, r] = max(q_r . kmax_i, q_r . kmin_i) for the M*G query rows r of the KV
 *   head (fp32 accumulation; or the channel-wise bound if cfg->score says so); score[i] = mean / max over all rows, or the mean
 *   over the G rows of tree->last_node;
 *   kept = blocks [0, ns) + the k best candidates of [ns, nb_b - nr) by (fp32
 *   score descending, block index ascending) + blocks [nb_b - nr, nb_b);
 *   every block if nb_b <= ns + k + nr.
 * sel_idx   [batch, Hkv, n_sel] int32, n_sel = ns + k + nr + n_extra_slots, ascending, padded with -1.
 * sel_count [batch, Hkv] int32.
 * scores    optional [batch, Hkv, max_blocks] fp32 (NULL: kept in the workspace).
 * workspace may be NULL when scores is given; the one-launch route of specpv_debug_set_select_route
 * uses the arrival words of a workspace of 64 KiB or more (zero before the call, zero again after it). */
int specpv_select_blocks(const specpv_kv *kv, const specpv_tree *tree,
                         const void *kmax, const void *kmin, const specpv_select_cfg *cfg,
                         int32_t *sel_idx, int32_t *sel_count, float *scores,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Section 3.2 (attention over the partial cache as one KV segment) with the tree
 * decode of Algorithm 1.  For node j and query head h (KV head g = h / G):
 *   keys = tokens t < L_b of the blocks sel_idx[b, g, 0..sel_count[b, g])
 *          + draft nodes a that are j or an ancestor of j;
 *   out[b, j, h, :] = softmax(q . k / sqrt(D)) . v over those keys (fp32
 *   accumulation, result in the q dtype); lse[b, j, h] = log sum exp (natural log).
 *   Only the Mq query nodes have rows in q, out and lse (row j - n_key_only).
 * sel_idx == NULL attends over every block (full verification).  The order of
 * sel_idx does not matter; entries < 0 or >= nb_b are ignored; a block listed
 * twice is attended twice.
 * out [batch, Mq, Hq, D]; lse optional [batch, Mq, Hq] fp32.
 * Value range (bf16, head dim 128): the context part is computed in several pieces whose
 * normalised results (convex combinations of V rows) travel through the workspace as fp16, so
 * V entries are assumed to lie within +-65504; larger magnitudes are clamped there, not reported. */
int specpv_partial_verify_attn(const specpv_kv *kv, const specpv_tree *tree,
                               const int32_t *sel_idx, const int32_t *sel_count, int32_t n_sel,
                               void *out, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream);

/* For callers that can neither allocate nor pass a workspace: code under HIP graph capture with
 * fixed arguments, tight serving loops, harnesses that forbid hipMalloc.  The same computation
 * as specpv_partial_verify_attn (same kernels, bit-identical results) with the split-KV partial
 * results kept in a file-scope device array of SPECPV_STATIC_SCRATCH_BYTES inside the library
 * (one copy per GPU, held until the process ends).  The call allocates nothing and calls no
 * allocating routine.  A call whose partial results would not fit (specpv_workspace_bytes with
 * cfg == NULL says how much a shape needs) returns SPECPV_ELIMIT, and specpv_last_hip_error()
 * then holds the two sizes; nothing has been enqueued.  Every call on a GPU shares that GPU's
 * array, which keeps the last call's contents; nothing in it needs to start at zero.  Calls that
 * overlap on one GPU (two streams without an ordering between them) race on it: order them. */
#define SPECPV_STATIC_SCRATCH_BYTES (16u << 20)
int specpv_partial_verify_attn_static(const specpv_kv *kv, const specpv_tree *tree,
                                      const int32_t *sel_idx, const int32_t *sel_count, int32_t n_sel,
                                      void *out, float *lse, void *stream);

/* Section 3.3: full verification that also refreshes the partial cache.
 *   1. summaries of blocks [stale_blk_begin, nb_b) are recomputed in place
 *      (stale_blk_begin < 0: none);
 *   2. attention of the tree over the whole cache -> out, lse;
 *   3. eq. 2 / eq. 3 scores with this pass's queries and a fresh selection
 *      -> sel_idx, sel_count (and scores if not NULL).
 * Same result as the three calls above issued one after another. */
int specpv_full_verify_refresh(const specpv_kv *kv, const specpv_tree *tree,
                               void *kmax, void *kmin, int32_t stale_blk_begin,
                               const specpv_select_cfg *cfg, void *out, float *lse,
                               int32_t *sel_idx, int32_t *sel_count, float *scores,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Section 3.2: the paper keeps the partial cache as a physically contiguous segment; this call
 * builds that variant from the kept-block lists (the attention calls above read the blocks in
 * place and do not need it).  For every sequence b and KV head g the tokens of the blocks
 * sel_idx[b, g, 0 .. sel_count[b, g]) are copied, in list order, to out_k / out_v
 * [batch, Hkv, n_sel * B, D] (same dtype; rows of list entries that are invalid or lie beyond
 * L_b are zero), and out_len[b] = the largest number of token rows any of its heads produced
 * (device, [batch]).  Attention over this gathered cache with sel_idx == NULL gives the same
 * result as attention over the lists when every head keeps the same number of full blocks. */
int specpv_gather_blocks(const specpv_kv *kv, const int32_t *sel_idx, const int32_t *sel_count, int32_t n_sel,
                         void *out_k, void *out_v, int32_t *out_len, void *stream);

/* ---- verification modes and the buffer (Section 3.3, Algorithm 1: SelectMode and the
 * KV side of PostEvaluate) ------------------------------------------------------------
 *
 * State of one sequence between verify steps: L committed tokens in the cache (all
 * fully verified) and n_pending partially verified tokens whose K/V wait in the
 * buffer for the next full verification.  The buffer is the K/V storage of the
 * (extended) draft tree: [batch, pending_cap + M_tree, Hkv, D], rows
 * pending_cap - n_pending .. pending_cap - 1 hold the pending tokens (oldest first),
 * rows pending_cap .. pending_cap + M_tree - 1 this step's candidates.  A verify step
 * then passes the rows from pending_cap - n_pending on as kd / vd of a tree with
 * n_pending + M_tree nodes whose parent array is a chain over the pending tokens with the
 * candidates' tree hanging off its end (specpv_extend_parents).  In a partial step the pending
 * tokens are keys only (tree.n_key_only = n_pending: no query rows); in a refresh step they are
 * queries as well (n_key_only = 0) and their K/V rows have been recomputed by the caller. */
typedef enum { SPECPV_MODE_FULL = 0, SPECPV_MODE_PARTIAL = 1, SPECPV_MODE_REFRESH = 2 } specpv_mode;

typedef struct specpv_policy {
    int32_t partial_budget_tokens; /* size of the partial cache without the buffer: (ns + k + nr) * B */
    int32_t pending_margin_tokens; /* the buffer holds one step's candidates plus this many pending
                                      tokens (Section 4.2 and Appendix D: 20)                        */
} specpv_policy;

/* Section 3.3, last paragraph but one; SelectMode of Algorithm 1.  Host only, no GPU work.
 *   seq_len <= partial_budget_tokens           -> FULL    (partial verification disabled)
 *   partial cache not initialised yet           -> FULL    (the caller refreshes the selection with it)
 *   n_pending > pending_margin_tokens           -> REFRESH (pending + candidates exceed the buffer)
 *   otherwise                                   -> PARTIAL
 * seq_len counts committed and pending tokens.  Returns the mode, or SPECPV_EINVAL. */
int specpv_select_mode(const specpv_policy *policy, int64_t seq_len, int32_t partial_ready, int32_t n_pending);

/* Parent array (host memory, n_pending + M_tree entries) of the extended tree described
 * above: out[i] = i - 1 for the pending chain, the candidates' roots get n_pending - 1. */
int specpv_extend_parents(const int32_t *tree_parent, int32_t M_tree, int32_t n_pending, int32_t *out);

/* The kept-block lists of one layer, as specpv_select_blocks / specpv_full_verify_refresh wrote
 * them: sel_idx [batch, Hkv, n_sel], sel_count [batch, Hkv] (device). */
typedef struct specpv_lists {
    int32_t *sel_idx, *sel_count;
    int32_t n_sel;
} specpv_lists;

/* Section 3.2 (the buffer holds the candidates' K/V until verification has decided which of
 * them survive) and Section 3.3 (after a full verification the rejected candidates leave both
 * caches).  accepted [batch, max_accept] int32 (device): the candidates on the accepted
 * path as indices 0 .. M_tree-1 in increasing order; n_accepted [batch] (device).
 *   mode PARTIAL: the accepted candidates' K/V rows join the pending tokens (the buffer is
 *     compacted: everything else of this step's candidates is dropped);
 *     n_pending_b += n_accepted_b, at most pending_cap.
 *   mode FULL / REFRESH: the pending tokens' rows, then the accepted candidates' rows, are
 *     appended to the cache at tokens L_b, L_b + 1, ...; L_b grows by their number, at most to
 *     max_blocks * B; n_pending_b = 0; the summaries (eq. 1) of every block that received a
 *     token are recomputed (kmax == NULL: skipped); and, as Section 3.3 has the local window
 *     follow the sequence's end, with lists != NULL every block that received a token joins each KV head's
 *     list behind its last entry unless it is that entry already (the ragged last block of the
 *     local window), so that the committed tokens stay visible to the partial steps that follow.
 *     A row of n_sel entries needs n_extra_slots >= ceil((pending_cap + max_accept) / B) + 1
 *     free ones for that.
 * Storage is finite: tokens are stored oldest first while the cache (or the buffer) has room.
 * dropped (device, [batch, 2] int32, may be NULL) receives what did not fit: [b, 0] the number
 * of tokens of sequence b that were NOT stored, [b, 1] the largest number of blocks that found
 * no free entry in a list row of sequence b.  Both are 0 unless the caller under-sized the
 * cache, the buffer or the list rows; a caller that cannot rule that out has to check them.
 * Writes through kv->k, kv->v (rows from L_b on; the allocation must cover max_blocks * B
 * tokens) and kv->ctx_len, n_pending [batch] (device), in stream order.  Workspace: 4 bytes
 * per sequence (specpv_workspace_bytes covers it). */
int specpv_commit_accepted(const specpv_kv *kv, void *buf_k, void *buf_v, int32_t pending_cap, int32_t M_tree,
                           int32_t *n_pending, const int32_t *accepted, const int32_t *n_accepted,
                           int32_t max_accept, specpv_mode mode, void *kmax, void *kmin,
                           const specpv_lists *lists, int32_t *dropped,
                           void *workspace, size_t workspace_bytes, void *stream);

/* The same for the n_layers layers of a model in one go (the accepted path is the same for every
 * layer of a verify step).  kv, buf_k, buf_v, kmax, kmin: HOST arrays of n_layers descriptors /
 * device pointers (kmax, kmin may be NULL, or arrays of NULLs, to skip the summaries); lists: a
 * HOST array of n_layers list descriptors with one n_sel, or NULL.  All
 * layers must share one shape, one set of strides, one dtype and ONE ctx_len array; the counters
 * (ctx_len, n_pending) are read by every layer's copies and updated once afterwards, so the
 * result is what specpv_commit_accepted would give per layer on private copies of the counters.
 * 1 <= n_layers <= SPECPV_MAX_LAYERS.  A few launches for up to 32 layers instead of a few per layer. */
#define SPECPV_MAX_LAYERS 256
int specpv_commit_accepted_layers(const specpv_kv *const *kv, void *const *buf_k, void *const *buf_v,
                                  int32_t n_layers, int32_t pending_cap, int32_t M_tree,
                                  int32_t *n_pending, const int32_t *accepted, const int32_t *n_accepted,
                                  int32_t max_accept, specpv_mode mode, void *const *kmax, void *const *kmin,
                                  const specpv_lists *lists, int32_t *dropped,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* Testing and measuring aid, process-wide (not per thread, not per stream): how
 * specpv_partial_verify_attn runs the shapes that its eight-wavefront kernel takes (bf16, head dim
 * 128, short token ranges).
 *   0  the library's choice (currently two kernels)
 *   1  two kernels: context attention, then the log-sum-exp combine with the draft-tree segment
 *   2  one kernel: the draft-tree segment is one more partial, and the last workgroup of a row
 *      tile to arrive merges the tile's partials out of its XCD's L2 (no workgroup waits for another)
 *   3  as 2, and the last workgroup of every tile takes the route that is otherwise only taken when
 *      workgroups of a tile ran on different XCDs: it recomputes the tile by itself
 * All give results within the documented bars.  Returns SPECPV_OK or SPECPV_EINVAL. */
int specpv_debug_set_route(int route);

/* Testing and measuring aid, process-wide: how specpv_select_blocks and the refresh of
 * specpv_full_verify_refresh run scoring + selection (Section 3.2, eq. 2-3 and the top-k).
 *   0  the library's choice (currently two launches)
 *   1  one launch where that is possible, two elsewhere: every scoring workgroup counts itself in on
 *      arrival words of its (sequence, KV head) at the head of the workspace, and the last one to
 *      arrive selects (no workgroup waits for another; the words are zero again afterwards).
 *      Possible where the matrix-core scoring kernel applies (bf16, head dim 128), the tree has more
 *      than 96 query rows per KV head, max_blocks <= 4096, batch * n_kv_heads <= 910 and the call
 *      has a workspace of 64 KiB or more
 *   2  two launches: scoring, then selection
 * Both give the same lists and scores, bit for bit.  Returns SPECPV_OK or SPECPV_EINVAL. */
int specpv_debug_set_select_route(int route);

/* Measuring aid, process-wide.  A library built with -DSPECPV_TIMELINE (`python -m paper_2512_02337_amd.build
 * --timeline` makes libspecpv_timeline.so) has every workgroup of the partial-verify attention kernel store 16
 * 64-bit readings of the 100 MHz real-time counter at fixed points of its course to
 * buf[(blockIdx.y * gridDim.x + blockIdx.x) * 16 + i] (device memory, 4096 rows of 16 words, NULL = off);
 * the combine kernel writes rows 2048 + workgroup, and rows 3072 + workgroup receive three words per attention
 * workgroup: core cycles (s_memtime), 10 ns ticks and chunks of its life, from which the core clock follows.
 * The kernel for long token ranges (full verification) writes only those three words, to row workgroup.
 * paper_2512_02337_amd/timeline.py names the points and prints their medians.  A regular build takes no
 * stamps and answers a non-NULL buf with SPECPV_EINVAL. */
int specpv_debug_set_timeline(void *buf);

const char *specpv_strerror(int status);
/* Text of the HIP error behind the calling thread's last SPECPV_EHIP. */
const char *specpv_last_hip_error(void);
int specpv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECPV_H */
