/*
 * seqtree -- the target model's verification step over a speculated token tree
 * (Sequoia, arxiv 2402.12374), as a C-ABI library for AMD MI355X (gfx950).
 *
 * Two operations make up the step:
 *   seq_tree_attn   one attention layer of the target model's one forward pass over the whole
 *                   tree, which scores all of its tokens together (Sec. 1; Sec. 2.1: the root
 *                   stands for the current prefix): tree token i attends to the prefix KV
 *                   cache, to its ancestors in the tree and to itself.
 *   seq_verify      Algorithm 2 (Sec. 3.2.1, "Sequoia Sampling and Verification") applied
 *                   recursively from the root (Sec. 2.2), on caller-supplied uniforms.
 * Around them:
 *   seq_draft_sample      the drafter's ordered draw of child tokens without replacement (Sec. 3.2.1, 4.1)
 *   seq_verify_with       the same walk with SpecInfer's or naive / top-k sampling's rule (Sec. 2.2)
 *   seq_verify_batched    the walk for several sequences that share the tree
 *   seq_build_tree, seq_tree_expected_tokens, seq_pick_tree_shape
 *                         Sequoia's tree construction and hardware-aware choice of size and depth
 *                         (Sec. 3.1.2, 4.1; host only)
 *   seq_top_p_filter, seq_kv_append
 *                         glue between two steps: nucleus filtering of logit rows; the accepted
 *                         path's K/V rows join the prefix
 *
 * Conventions for every entry point
 *   - Tensors are row-major and contiguous.  Pointers are DEVICE pointers unless marked HOST.
 *   - The caller owns every buffer.  Inputs are never written.  The library keeps, per
 *     process, a cache of tree plans (device copies of the ancestor bitset and the child lists,
 *     keyed by the device and the contents of parent[]; 1 KB at 64 nodes, 140 KB at 1024) and one
 *     synchronisation area (8.3 MiB) per (device, stream) it has been called on; both are created
 *     on first use and released by seq_shutdown() only.  Nothing is ever evicted -- a captured
 *     graph holds the device pointers of the plan and the area it was captured with -- so at most
 *     SEQ_MAX_PLANS distinct trees and SEQ_MAX_STREAMS streams per device can be in use between
 *     two seq_shutdown() calls; one more is refused with SEQ_ERR_FULL.
 *   - The first call for a tree, and the first call on a stream, allocates device memory and
 *     copies synchronously.  Every later call with that tree on that stream allocates nothing,
 *     copies nothing and never synchronises with the host.  Under stream capture nothing can be
 *     allocated: a call with a tree that is not cached yet is refused (SEQ_ERR_CAPTURE), and a
 *     capturing stream that has no area yet records its calls with the area of the first stream
 *     the library was called on for this device (SEQ_ERR_CAPTURE if there is none): make one
 *     call with the tree outside capture first.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default
 *     stream); outputs are valid once the caller has synchronised that stream.
 *   - Return value: SEQ_OK (0) or a negative SEQ_ERR_* code.  Nothing is thrown or printed.
 *     All argument checks happen on the host before any GPU call, so invalid arguments are
 *     reported even on a machine without a GPU.
 *   - Calls on different streams may overlap in time: each stream has its own synchronisation
 *     area, and calls on one stream are ordered by the stream.  A captured graph keeps the area
 *     it was recorded with wherever it is replayed: do not replay it while other work that uses
 *     that area (eager calls on the stream the area belongs to, another graph recorded with it)
 *     may be running.  seq_shutdown() must not run while any call or graph is in flight.
 */
#ifndef SEQTREE_H
#define SEQTREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of q/k/v/out and of the logits */
#define SEQ_BF16 1
#define SEQ_F32 2

#define SEQ_OK 0
#define SEQ_ERR_NULL (-1)        /* a required pointer is NULL */
#define SEQ_ERR_SHAPE (-2)       /* n_tree < 1 or > SEQ_MAX_TREE, head_dim not 64/128, heads % kv_heads != 0,
                                    prefix_len < 0 or > prefix_cap, vocab < 2 or > SEQ_MAX_VOCAB */
#define SEQ_ERR_TREE (-3)        /* parent[0] != -1 or parent[i] not in [0, i) */
#define SEQ_ERR_DTYPE (-4)       /* dtype is neither SEQ_BF16 nor SEQ_F32 */
#define SEQ_ERR_TEMPERATURE (-5) /* temperature negative, NaN or infinite */
#define SEQ_ERR_WORKSPACE (-6)   /* workspace NULL, smaller than the matching *_workspace(), or not 16-byte aligned */
#define SEQ_ERR_HIP (-7)         /* a HIP runtime call failed (no device, launch failure, ...) */
#define SEQ_ERR_ALGORITHM (-8)   /* algorithm is none of SEQ_VERIFY_* */
#define SEQ_ERR_FULL (-9)        /* SEQ_MAX_PLANS distinct trees or SEQ_MAX_STREAMS streams are already in use */
#define SEQ_ERR_CAPTURE (-10)    /* under stream capture: first call for this tree, or first call on this device */
#define SEQ_ERR_ALIGN (-11)      /* seq_tree_attn*: q, k/v cache, k/v tree or out not 16-byte aligned */

#define SEQ_MAX_TREE 1024
#define SEQ_MAX_VOCAB 524288
#define SEQ_MAX_CHILDREN 64      /* most tokens seq_draft_sample draws for one node */
#define SEQ_MAX_PLANS 1024       /* distinct (device, tree) pairs the plan cache holds */
#define SEQ_MAX_STREAMS 16       /* streams per device with a synchronisation area of their own */

/*
 * Tree-masked attention with grouped-query heads (one layer).
 *
 * For query head h (KV head g = h / (heads / kv_heads)) and tree token i:
 *     keys(i)      = cache rows 0..prefix_len-1  u  tree rows j with j == i or j an ancestor of i
 *     out[i,h,:]   = softmax_x( <q[i,h,:], k_x[g,:]> / sqrt(head_dim) ) . v_x[g,:]   over x in keys(i)
 * Every other key has weight exactly zero (its K/V rows may hold anything, NaN included).
 * Positional encodings, if any, are applied by the caller beforehand.
 *
 *   q        [n_tree, heads, head_dim]
 *   k_cache  [kv_heads, prefix_cap, head_dim]   first prefix_len rows of each head are valid
 *   v_cache  same layout
 *   k_tree   [n_tree, kv_heads, head_dim]       row 0 belongs to the root (the last accepted
 *   v_tree   same layout                         token, whose K/V is not yet in the cache)
 *   parent   HOST [n_tree]; parent[0] = -1; 0 <= parent[i] < i
 *   out      [n_tree, heads, head_dim], same dtype as the inputs
 *   dtype    SEQ_BF16 (bf16 MFMA, fp32 accumulation) or SEQ_F32 (fp32 throughout)
 *   workspace, workspace_bytes   scratch of at least seq_tree_attn_workspace(...) bytes
 *
 * All six tensors are DEVICE memory and 16-byte aligned (the kernels move them 16 bytes at a
 * time; SEQ_ERR_ALIGN otherwise).
 * prefix_len = 0 (tree only) and n_tree = 1 (plain decode attention) are legal.
 *
 * A batch of B sequences that share the tree and the prefix length is one call with
 * heads = B * H and kv_heads = B * Hk on tensors laid out q, out [n_tree, B, H, head_dim],
 * k_tree, v_tree [n_tree, B, Hk, head_dim], k_cache, v_cache [B, Hk, prefix_cap, head_dim]:
 * query head b * H + h uses KV head b * Hk + h / (H / Hk), so a sequence sees only its own rows.
 */
int seq_tree_attn(const void* q, const void* k_cache, const void* v_cache,
                  const void* k_tree, const void* v_tree, const int32_t* parent,
                  int32_t prefix_len, int32_t n_tree, int32_t heads, int32_t kv_heads,
                  int32_t head_dim, void* out,
                  int32_t prefix_cap, int32_t dtype,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Verification walk (Algorithm 2 at every node on the way down, Sec. 3.2.1 / Sec. 2.2).
 *
 * With P_v = softmax(target_logits[v,:] / T) and Q_v = softmax(draft_logits[v,:] / T):
 *     v = root;  loop:
 *       R = P_v, D = Q_v, S = {}
 *       for each child c of v in ascending node id (the order the drafter sampled them):
 *           s = tree_tokens[c];  accept c iff uniforms[c] < R[s] / D[s]   (strict)
 *           accepted: append c to accepted_path, v = c, restart the loop
 *           rejected: R = norm(max(R - D, 0));  D[s] = 0;  S += s;
 *                     if sum(D) == 0: D = uniform over tokens not in S;  D = norm(D)
 *       no child accepted: bonus_token ~ R by inverse CDF over ascending token id using
 *           uniforms[0] (first x with inclusive cumulative mass > u * sum(R));  stop.
 * T = 0 is greedy: P and Q are one-hot at the arg-max (lowest index on ties), which reduces
 * the walk to "accept c iff tree_tokens[c] == argmax target_logits[v]".
 * A token with D[s] = 0 is accepted iff R[s] > 0.
 *
 *   target_logits  [n_tree, vocab]   row v: the target's next-token logits after node v
 *   draft_logits   [n_tree, vocab]   row v: the draft logits v's children were sampled from
 *   tree_tokens    [n_tree] int32    token id of node i, in [0, vocab); entry 0 is ignored
 *   parent         HOST [n_tree]
 *   temperature    >= 0, finite
 *   uniforms       [n_tree] float in [0,1): [i >= 1] decides node i, [0] draws the bonus token
 *   accepted_path  [n_tree] int32 out: accepted node ids from the root's child downwards,
 *                  every remaining entry -1
 *   bonus_token    [1] int32 out
 *   workspace      DEVICE, 16-byte aligned, at least seq_verify_workspace(...) bytes; on return it
 *                  starts with a trace (see below) that tests and debuggers may read; the rest
 *                  is scratch whose contents are unspecified.  It need not be cleared: nothing
 *                  it holds on entry is read (what workgroups hand to each other travels
 *                  through the stream's synchronisation area).
 *
 * Three kernels sit behind this call and give the same results.  For sampling (T > 0) every
 * node's accept thresholds can be computed at once and a short walk follows: over a vocabulary
 * of at most 32768 tokens with one workgroup per node (every logit row the tree can visit is
 * read), for trees of at most 256 nodes; over larger vocabularies with a team of
 * ceil(vocab / 16384) workgroups per node that has children, while every member finds a compute
 * unit of its own (a 64-node tree over 128256 tokens: 32 teams of 8).  Otherwise only the rows
 * of the nodes the walk visits are read, by workgroups that share the vocabulary.
 */
int seq_verify(const void* target_logits, const void* draft_logits,
               const int32_t* tree_tokens, const int32_t* parent, float temperature,
               const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
               int32_t n_tree, int32_t vocab, int32_t dtype,
               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same walk with one of the baseline verification algorithms of Sec. 2.2 at every node
 * (seq_verify is seq_verify_with(SEQ_VERIFY_SEQUOIA, ...)).  Arguments, outputs, workspace and
 * errors as for seq_verify; SEQ_ERR_ALGORITHM for an unknown algorithm.
 *
 *   SEQ_VERIFY_SPECINFER  Algorithm 2 without its blue lines: the children are taken to be
 *       independent draws from the draft distribution, which therefore stays what it was after a
 *       rejection (no token is struck out, nothing is renormalised, repeated tokens are legal):
 *       accept c iff uniforms[c] < R[s] / Q[s];  rejected: R = norm(max(R - Q, 0)).
 *   SEQ_VERIFY_TOPK       naive / top-k sampling: at the node v the walk stands on, draw
 *       x ~ softmax(target_logits[v] / T) by inverse CDF with uniforms[v] (the root: uniforms[0]);
 *       if x is the token of a child of v, the first such child in sibling order is accepted and
 *       the walk goes on there; otherwise bonus_token = x and the walk ends.  draft_logits is not
 *       read and may be NULL.  Every node's draw is computed (one workgroup per node), then the
 *       walk follows them.
 * At temperature 0 all three accept a child exactly when its token is the arg-max of the
 * target's row and emit that arg-max.
 * Trace: as below for SPECINFER.  For TOPK one record per visited node: int32 node, int32 accepted
 * child or -1, int32 drawn token, float uniform; header [3], [4] are zero; the four floats about
 * the bonus draw describe the last draw.
 */
#define SEQ_VERIFY_SEQUOIA 0
#define SEQ_VERIFY_SPECINFER 1
#define SEQ_VERIFY_TOPK 2
int seq_verify_with(int32_t algorithm, const void* target_logits, const void* draft_logits,
                    const int32_t* tree_tokens, const int32_t* parent, float temperature,
                    const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
                    int32_t n_tree, int32_t vocab, int32_t dtype,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The walk for a batch of sequences that share the tree: every array of seq_verify_with gains a
 * leading dimension `batch` (logits [batch, n_tree, vocab], tree_tokens, uniforms, accepted_path
 * [batch, n_tree], bonus_token [batch]); parent stays one tree.  The workspace is batch times
 * seq_verify_workspace(...) bytes, sequence b's trace starting at byte b * seq_verify_workspace(...).
 * batch 1 .. 256.  Sequences share launches: floor(256 / n_tree) of them where the per-node
 * kernel applies and the batch fits in as few launches that way, otherwise the lazy walk with the
 * teams of min(64, floor(256 / W)) sequences side by side, W = ceil(vocab / 8192) workgroups per
 * team; SEQ_VERIFY_TOPK at temperature > 0 runs the whole batch in one launch per kernel.  A team
 * that times out waiting for its members reports status 1 in its own sequence's trace.
 */
int seq_verify_batched(int32_t algorithm, int32_t batch, const void* target_logits, const void* draft_logits,
                       const int32_t* tree_tokens, const int32_t* parent, float temperature,
                       const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
                       int32_t n_tree, int32_t vocab, int32_t dtype,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Trace left at the start of the seq_verify workspace.  Header of 8 int32:
 *   [0] number of accept tests recorded   [1] status: 0 ok, 1 = the cooperating workgroups
 *   timed out waiting for each other (outputs invalid)   [2] node the bonus token was drawn at
 *   [3] number of uniform fallbacks   [4] number of degenerate residual updates   [5..7] zero
 * followed by one record of 4 x 32 bit per accept test, in order:
 *   int32 node, int32 accepted (0/1), float ratio R[s]/D[s], float uniform
 * and after SEQ_MAX_TREE such records 4 floats about the bonus draw:
 *   u, sum(R) before normalisation by the residual mass, cumulative mass below the drawn
 *   token, cumulative mass including it (the last three relative to sum(R) = 1).
 */
#define SEQ_TRACE_HEADER_INTS 8
#define SEQ_TRACE_RECORD_WORDS 4

/*
 * The drafter's ordered draw of child tokens without replacement -- the sampling half of
 * Algorithm 2 (Sec. 3.2.1: children are drawn without replacement from the draft distribution,
 * and uniformly from the tokens not drawn yet once its support is used up), by the
 * exponential-sort method the implementation details name (Sec. 4.1).
 *
 * For every row r and token x:
 *     word  = output word x % 4 of Philox4x32-10 with key (seed low, seed high) and
 *             counter (x / 4, r, step low, step high)
 *     w     = ((word >> 9) + 0.5) * 2^-23                    uniform in (0,1)
 *     key   = draft_logits[r,x] / temperature - ln(-ln w)    (exponential sort, in logarithms)
 * and tokens[r, 0 .. n_children[r]) are the tokens of the n_children[r] largest keys in
 * descending order of key (lower id first among equal keys), the rest of the row -1.  Tokens of
 * zero probability (logit -inf or NaN, or logit / temperature below -2^103) come after all
 * others, in descending order of -ln(-ln w) alone, i.e. uniformly at random.
 * temperature = 0 is the limit T -> 0+: the n_children[r] largest logits in descending order,
 * lower id first among equals (top-k drafting, Sec. 2.2); seed and step are not read.
 * Keys are computed in fp32; two keys closer than a few 1e-6 may come out in either order.
 *
 *   draft_logits  [n_rows, vocab]   one row per node whose children are drawn now
 *   n_children    DEVICE [n_rows] int32, each in [0, k_max] (values outside are clamped)
 *   rng           DEVICE [2] uint64: seed, step.  It lives on the device so that a captured
 *                 graph draws fresh numbers on every replay once the caller has advanced step.
 *   tokens        [n_rows, k_max] int32 out
 *   n_rows        1 .. SEQ_MAX_TREE;  vocab 2 .. SEQ_MAX_VOCAB;  k_max 1 .. min(SEQ_MAX_CHILDREN, vocab)
 *   workspace     DEVICE, 16-byte aligned, at least seq_draft_sample_workspace(...) bytes; scratch
 *                 (reserved: the current kernel keeps everything in registers and in the
 *                 library's per-device exchange area)
 *
 * Errors: SEQ_ERR_NULL, SEQ_ERR_DTYPE, SEQ_ERR_SHAPE, SEQ_ERR_TEMPERATURE, SEQ_ERR_WORKSPACE,
 * SEQ_ERR_HIP.  One launch.  Rows that several workgroups share meet in the stream's
 * synchronisation area.
 */
int seq_draft_sample(const void* draft_logits, const int32_t* n_children, float temperature,
                     const uint64_t* rng, int32_t* tokens, int32_t n_rows, int32_t vocab,
                     int32_t k_max, int32_t dtype, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/*
 * Appends the K/V rows of the root and of the accepted tree nodes to the cache, in path order:
 * row prefix_len of every head receives node 0's, row prefix_len + j the j-th accepted node's
 * (loop glue between two steps; not described in the paper, whose KV cache lives inside the
 * Transformers library).  The next step runs with the new prefix length and a new tree.
 *
 *   k_tree, v_tree   [n_tree, kv_heads, head_dim]   this step's tree tensors
 *   accepted_path    DEVICE [n_tree] int32, as seq_verify leaves it (node ids, then -1)
 *   parent           HOST [n_tree]: bounds the path length (the tree's depth)
 *   k_cache, v_cache [kv_heads, prefix_cap, head_dim], written in place at rows >= prefix_len
 *   new_prefix_len   DEVICE [1] out, may be NULL: prefix_len + 1 + number of accepted nodes
 * Rows that would fall at or beyond prefix_cap are not written and new_prefix_len stops at
 * prefix_cap: the caller sizes the cache for prefix_len + depth + 1.  A path entry that is not a
 * node id ends the path.  Pointers 16-byte aligned.  Asynchronous on hip_stream, no host sync.
 * Errors: SEQ_ERR_NULL, SEQ_ERR_DTYPE, SEQ_ERR_SHAPE, SEQ_ERR_TREE, SEQ_ERR_HIP.
 */
int seq_kv_append(const void* k_tree, const void* v_tree, const int32_t* accepted_path,
                  const int32_t* parent, void* k_cache, void* v_cache, int32_t prefix_len,
                  int32_t n_tree, int32_t kv_heads, int32_t head_dim, int32_t prefix_cap,
                  int32_t dtype, int32_t* new_prefix_len, void* hip_stream);

/*
 * Nucleus (top-p) filtering of logit rows, the sampling hyper-parameter of the paper's table on
 * robustness to top-p (appendix "Robustness additional results"): of softmax(logits / temperature)
 * the most probable tokens are kept, as few as reach a total probability of top_p (equal
 * probabilities at the cut: lower token id first); every other logit becomes -inf, which
 * seq_verify and seq_draft_sample read as probability zero.  Kept logits are copied unchanged.
 * temperature 0: only the arg-max (lowest id) is kept.  top_p = 1: every token whose fp32
 * probability is not zero is kept.  NaN reads as -inf.
 *
 *   logits    [n_rows, vocab];  filtered  [n_rows, vocab] out, may be the same buffer
 *   top_p     in (0, 1];  n_rows 1 .. SEQ_MAX_TREE;  vocab 2 .. SEQ_MAX_VOCAB
 *   kept      DEVICE [n_rows] int32 out, may be NULL: tokens kept per row
 * Probabilities are fp32 (sums in fp64): a cut that falls within about 1e-6 of top_p, or between
 * tokens whose probabilities agree to fp32 precision, may keep one token more or fewer than exact
 * arithmetic.  One workgroup per row; rows above 32768 tokens are re-read from cache at each of the
 * 30 bisection steps (slow).  Errors: SEQ_ERR_NULL, SEQ_ERR_DTYPE, SEQ_ERR_SHAPE (top_p outside
 * (0, 1] included), SEQ_ERR_TEMPERATURE, SEQ_ERR_HIP.
 */
int seq_top_p_filter(const void* logits, void* filtered, float top_p, float temperature,
                     int32_t n_rows, int32_t vocab, int32_t dtype, int32_t* kept, void* hip_stream);

/*
 * seq_tree_attn for a batch of sequences that share the tree but not the prefix length (the
 * paper's limitations section: serving means batches; sequences of a batch have histories of
 * different lengths).  Sequence b attends to the first prefix_lens[b] cache rows of its own KV
 * heads and to the tree; otherwise the definition above, per sequence.
 *
 *   q, out       [n_tree, batch, heads, head_dim]
 *   k_tree, v_tree   [n_tree, batch, kv_heads, head_dim]
 *   k_cache, v_cache [batch, kv_heads, prefix_cap, head_dim]
 *   parent       HOST [n_tree], one tree for the whole batch
 *   prefix_lens  DEVICE [batch] int32.  It is read by the kernel, not by the host, so a captured
 *                call follows the lengths as the caller updates them between replays.
 *   max_prefix_len   HOST: a bound on every prefix_lens[b], at most prefix_cap; the work is cut
 *                for this length (a length beyond it is read as max_prefix_len, a negative one as 0)
 *   heads, kv_heads  per sequence;  batch 1 .. SEQ_MAX_BATCH
 *   workspace    at least seq_tree_attn_batched_workspace(...) bytes
 * Errors as for seq_tree_attn.
 */
#define SEQ_MAX_BATCH 4096
int seq_tree_attn_batched(const void* q, const void* k_cache, const void* v_cache,
                          const void* k_tree, const void* v_tree, const int32_t* parent,
                          const int32_t* prefix_lens, int32_t max_prefix_len, int32_t batch,
                          int32_t n_tree, int32_t heads, int32_t kv_heads, int32_t head_dim,
                          void* out, int32_t prefix_cap, int32_t dtype,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
size_t seq_tree_attn_batched_workspace(int32_t max_prefix_len, int32_t batch, int32_t n_tree, int32_t heads,
                                       int32_t kv_heads, int32_t head_dim, int32_t dtype);

/*
 * seq_tree_attn for callers that cannot allocate device memory: code under stream capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments (no workspace), same kernels,
 * same results bit for bit.  The call allocates nothing, frees nothing, copies nothing between
 * host and device and looks nothing up: the ancestor bitset is rebuilt on the device at every call
 * from parent[], which travels as a kernel argument, and bitset, arrival counters and partial
 * results live in one static device array of 192 KiB + SEQ_NOALLOC_MAX_PARTIAL_BYTES that every
 * GPU the library runs on holds until the process ends.
 *
 * Limits: n_tree <= SEQ_MAX_TREE as everywhere; a shape whose key ranges need more than
 * SEQ_NOALLOC_MAX_PARTIAL_BYTES of partial results (seq_tree_attn_workspace(...) says how much) is
 * refused with SEQ_ERR_WORKSPACE.  Other errors as for seq_tree_attn.
 *
 * All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in time
 * on one GPU race; order them (one stream, or events).  The array keeps the last call's contents;
 * what a call needs cleared it clears itself, on its stream.  The first call on each GPU finds the
 * array's address and measures how the GPU places workgroups (a small kernel on the null stream
 * and a synchronous read-back): make it outside stream capture (SEQ_ERR_CAPTURE otherwise).
 */
#define SEQ_NOALLOC_MAX_PARTIAL_BYTES (32u << 20)
int seq_tree_attn_noalloc(const void* q, const void* k_cache, const void* v_cache,
                          const void* k_tree, const void* v_tree, const int32_t* parent,
                          int32_t prefix_len, int32_t n_tree, int32_t heads, int32_t kv_heads,
                          int32_t head_dim, void* out, int32_t prefix_cap, int32_t dtype,
                          void* hip_stream);

/* Scratch sizes in bytes for the calls above (0 is never returned; at least 256). */
size_t seq_tree_attn_workspace(int32_t prefix_len, int32_t n_tree, int32_t heads,
                               int32_t kv_heads, int32_t head_dim, int32_t dtype);
size_t seq_verify_workspace(int32_t n_tree, int32_t vocab, int32_t dtype);
size_t seq_draft_sample_workspace(int32_t n_rows, int32_t vocab, int32_t k_max, int32_t dtype);

/*
 * Host-only helper: the tree plan both calls derive from parent[] (no GPU involved).
 *   depth        [n_tree]      depth[0] = 0
 *   child_start  [n_tree + 1]  children of v are child_list[child_start[v] .. child_start[v+1])
 *   child_list   [n_tree - 1]  ascending node id within each sibling list = drafting order
 *   anc_words    [n_tree * words_per_row] uint32, words_per_row = 2 * ceil(n_tree / 64):
 *                bit j of row i is set iff j == i or j is an ancestor of i
 * Any output pointer may be NULL.  Returns SEQ_OK, SEQ_ERR_SHAPE or SEQ_ERR_TREE.
 */
int seq_tree_plan_host(const int32_t* parent, int32_t n_tree, int32_t* depth,
                       int32_t* child_start, int32_t* child_list, uint32_t* anc_words);

/*
 * Sequoia tree construction (Sec. 3.1.2, Algorithm 1 with the depth bound of its appendix).  HOST
 * only, no GPU involved; meant to run once, ahead of time.
 *
 * acceptance[k-1] is the probability that the token at child position k of an accepted node is
 * accepted (the acceptance vector).  The expected number of tokens one verification of a tree
 * generates is F = sum over its nodes of the product of the rates along the node's path (root: 1).
 * seq_build_tree returns a tree of exactly n_tree nodes, at most max_branch children per node
 * and depth at most max_depth (edges below the root) that maximises F, as a parent array in the
 * order the other calls expect: parent[0] = -1, parent[i] < i, breadth-first, the children of a
 * node in ascending id = child positions 1, 2, ... (the order they are drafted in).
 *
 *   acceptance       HOST [max_branch], each in [0, 1];  max_branch 1 .. SEQ_MAX_CHILDREN
 *   n_tree           1 .. SEQ_MAX_TREE;  max_depth >= 0
 *   parent           HOST out [n_tree]
 *   expected_tokens  HOST out, may be NULL: F of the returned tree
 * Returns SEQ_ERR_SHAPE if no tree of that size exists within the bounds (or a rate is outside
 * [0, 1]).  Cost: n_tree^2 * max_depth * max_branch / 2 multiply-adds, 8 * n_tree * max_depth *
 * max_branch bytes (1024 nodes, 32 levels, 64 branches: about a second, 17 MB).
 */
int seq_build_tree(const double* acceptance, int32_t max_branch, int32_t n_tree, int32_t max_depth,
                   int32_t* parent, double* expected_tokens);

/* F of a given tree (HOST only): the closed form of Sec. 3.1.2.  Children beyond position
 * max_branch count with rate 0. */
int seq_tree_expected_tokens(const int32_t* parent, int32_t n_tree, const double* acceptance,
                             int32_t max_branch, double* expected_tokens);

/*
 * The hardware-aware choice of tree size and depth (Sec. 4.1), HOST only: over the given sizes n
 * and every depth d <= max_depth, maximise
 *     Speedup(n, d) = G(n, d) / (t(n) + d * c),
 * G(n, d) = F of the best tree of n nodes and depth <= d, t(n) = verify_time[i] / decode_time (the
 * target's time to verify n tokens relative to decoding one), c = draft_time / decode_time (one
 * draft step relative to the same).  Times are in any one unit, > 0 (draft_time may be 0).
 *   sizes, verify_time   HOST [n_sizes]: tree sizes (1 .. SEQ_MAX_TREE) and the measured time of
 *                        the target's forward pass over a tree of that size
 *   best_size, best_depth, best_speedup   HOST out (best_speedup may be NULL)
 */
int seq_pick_tree_shape(const double* acceptance, int32_t max_branch, const int32_t* sizes,
                        const double* verify_time, int32_t n_sizes, int32_t max_depth,
                        double decode_time, double draft_time, int32_t* best_size,
                        int32_t* best_depth, double* best_speedup);

/* Releases the plan cache and every synchronisation area (all devices, all streams).  Safe to call
 * twice.  Graphs captured before it hold dangling pointers afterwards and must not be replayed. */
int seq_shutdown(void);

const char* seq_strerror(int code);
int seq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SEQTREE_H */
