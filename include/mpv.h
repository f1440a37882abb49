/*
 * mpv.h -- batched lossless multi-path verification of draft token trees on one
 * AMD MI355X (gfx950).  C ABI; no C++ or PyTorch types cross this boundary.
 *
 * The operation (paper Sec. 2, step 3 "Verification"): for each of B draft trees
 * that share one shape, given the target and draft logits of every node, accept
 * one node of the tree and draw one correction ("bonus") token so that the
 * emitted tokens follow the target model's distribution.
 *
 * Tree (Sec. 3, Def. 3.1; Sec. 3.2 root expansion; Sec. 5, Def. 5.2 delayed
 * expansion): node 0 is the root (the current context; it has logits but no
 * token).  parent[n] < n is the parent of node n >= 1.  The ordered child list
 * of a node is its children in ascending node index.  Sibling tokens are assumed
 * to be i.i.d. draws from the draft distribution of their parent; equal tokens
 * under one parent are separate nodes with separate rows.
 *
 * Node distributions (Sec. 3; Sec. 4.1 temperatures): p = softmax(z_target / T),
 * q = softmax(z_draft / T) over the full vocabulary, the same T for both.
 *
 * Methods:
 *   MPV_METHOD_SPECINFER  top-down walk of Sec. 3.2 with the SpecInfer solver of
 *                         App. B, Alg. 4 (children tried in list order; a child x
 *                         is accepted with min(1, p(x)/q(x)), otherwise
 *                         p <- normalise((p - q)_+)); when no child is accepted the
 *                         bonus token is drawn from the current p.
 *   MPV_METHOD_TRAVERSAL  bottom-up Traversal Verification (Sec. 3.2), with the
 *                         block-verification weights of Sec. 3.1:
 *                         w(child) = min(1, w(node) * P(x)/q(x)); leaves are tested
 *                         first in depth-first order; when a whole child subtree
 *                         is rejected the node's weight a and distribution P become
 *                         S/(S+1-a) and (a*P - q)_+/S with S = sum (a*P - q)_+.
 *                         The root is always accepted when reached.
 *   MPV_METHOD_NSS        top-down walk of Sec. 3.2 with the NSS solver of App. B,
 *                         Alg. 1: at every node a token is drawn from p; if it is
 *                         the token of a child the walk moves there (to the first
 *                         such child in list order), otherwise it ends and the
 *                         drawn token is the bonus token.  Draft logits are unused.
 *   MPV_METHOD_NAIVE      the same walk with the Naive solver of App. B, Alg. 2: the
 *                         first child x is accepted with min(1, p(x)/q(x)); otherwise
 *                         a token is drawn from (p - q)_+ and followed as above.
 *   MPV_METHOD_SPECTR     the same walk with the SpecTr solver (K-SEQ) of App. B, Alg. 3:
 *                         with rho* the root of 1 - (1 - beta(rho))^k = rho beta(rho) on [1,k],
 *                         beta(rho) = sum min(p/rho, q), the children are tested in list order
 *                         with min(1, p(x)/(rho* q(x))); otherwise a token is drawn from
 *                         (p - gamma min(p/rho*, q))_+, gamma = (1 - (1 - beta)^k)/beta, which at
 *                         rho* (where gamma = rho*) is (p - rho* q)_+.  The equation is solved in the
 *                         form sum (p - rho q)_+ = (sum (q - p/rho)_+)^k, the same numbers without
 *                         cancellation, by Newton's method to a relative 3e-8.
 *
 * Randomness: the caller supplies one uniform in [0,1) per node and tree.
 * uniforms[b,n] (n >= 1) is used only by the test of node n ("accept iff u < a");
 * uniforms[b,0] draws the bonus token by inverse CDF in vocabulary order
 * (smallest t whose cumulative residual mass exceeds u times the total).
 * NSS, NAIVE and SPECTR draw a token at every node they visit: the draw at node n uses
 * draw_uniforms[b,n], a second array of the same shape.
 *
 * All calls are thread-compatible, not thread-safe per stream.  No call
 * allocates or frees device memory or synchronises the device.
 */
#ifndef MPV_H
#define MPV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MPV_ABI_VERSION 9

/* limits (larger requests return MPV_ERR_UNSUPPORTED) */
#define MPV_MAX_NODES    64   /* nodes per tree, root included            */
#define MPV_MAX_CHILDREN 16   /* children of one node                      */
#define MPV_MAX_VOCAB    (1 << 21)
/* and B * (N + 2) <= 2^30 */

#define MPV_METHOD_SPECINFER 0
#define MPV_METHOD_TRAVERSAL 1
#define MPV_METHOD_NSS       2
#define MPV_METHOD_NAIVE     3
#define MPV_METHOD_SPECTR    4

#define MPV_DTYPE_F32  0      /* IEEE binary32 logits                      */
#define MPV_DTYPE_BF16 1      /* bfloat16 logits (upper half of binary32).  Finite values must lie
                               * within +-65504; magnitudes below 2^-14 are used to within 2^-25
                               * (an error of log2(e)/T * 2^-25 in the exponent of e^(z/T): nothing
                               * for T >= 0.01).  -inf marks a token of probability zero.        */

/* error codes: 0 = success, negative = failure (nothing was launched unless the
 * code is MPV_ERR_HIP, in which case some kernels may already be enqueued) */
#define MPV_OK                   0
#define MPV_ERR_NULL            -1   /* a required pointer is NULL                   */
#define MPV_ERR_BAD_SHAPE       -2   /* B < 0, N < 1, V < 1, max_depth < tree depth   */
#define MPV_ERR_BAD_TREE        -3   /* parent[0] != -1 or parent[n] not in [0, n)    */
#define MPV_ERR_BAD_TEMPERATURE -4   /* T is not a finite number > 0                  */
#define MPV_ERR_BAD_METHOD      -5
#define MPV_ERR_BAD_DTYPE       -6
#define MPV_ERR_WORKSPACE       -7   /* workspace NULL, misaligned or too small       */
#define MPV_ERR_UNSUPPORTED     -8   /* beyond MPV_MAX_*; stats / edge_probs with methods >= 2;
                                        acceptance rates of MPV_METHOD_TRAVERSAL        */
#define MPV_ERR_HIP             -9   /* a HIP call failed; see mpv_last_hip_error()   */
#define MPV_ERR_ALIGNMENT      -10   /* a logit base pointer is not 16-byte aligned   */
#define MPV_ERR_BAD_TOP_P      -11   /* top_p is not in (0, 1]                        */

/* Problem description.  Host memory, read during the call only. */
typedef struct mpv_problem {
    int32_t B;              /* trees in the batch (0 is allowed: nothing to do)      */
    int32_t N;              /* nodes per tree, root included                         */
    int32_t V;              /* vocabulary size                                       */
    int32_t method;         /* MPV_METHOD_*                                          */
    int32_t logit_dtype;    /* MPV_DTYPE_*                                           */
    float   temperature;    /* T > 0, applied to target and draft rows alike         */
    int32_t max_depth;      /* row width of path_nodes / path_tokens, >= tree depth  */
    const int32_t* parent;  /* HOST pointer, length N, shared by all trees           */
} mpv_problem;

/* Device buffers, all caller-owned, borrowed until the enqueued work has run.
 * Row-major, innermost index contiguous. */
typedef struct mpv_buffers {
    /* inputs */
    const void*    target_logits;  /* [B,N,V] of logit_dtype; every row may be read           */
    const void*    draft_logits;   /* [B,N,V] of logit_dtype; rows of leaves are never read   */
    const int32_t* tokens;         /* [B,N]; tokens[b,0] ignored; others in [0,V)             */
    const float*   uniforms;       /* [B,N] in [0,1)                                          */
    /* outputs */
    int32_t*  accept_len;          /* [B]   depth tau of the accepted node                    */
    int32_t*  path_nodes;          /* [B,max_depth] node indices root-to-accepted, -1 padded  */
    int32_t*  path_tokens;         /* [B,max_depth] their tokens, -1 padded                   */
    int32_t*  bonus_token;         /* [B]   the correction token                              */
    uint32_t* counters;            /* [MPV_COUNTER_COUNT] see MPV_COUNTER_*; zeroed by the call */
    /* optional debug outputs (NULL = not wanted) */
    float* stats;                  /* [B,N,4] m_t, logZ_t, m_d, logZ_d: row maximum and
                                      ln sum exp((z-m)/T); draft entries of leaves are NaN    */
    float* edge_probs;             /* [B,N,2] p(x_n), q(x_n) under the parent's softmax; n=0: 1,1 */
    float* accept_prob;            /* [B,N] probability node n is tested with when reached; n=0: 1 */
    float* final_residual;         /* [B,V] normalised distribution the bonus token is drawn from */
    /* input of MPV_METHOD_NSS, MPV_METHOD_NAIVE and MPV_METHOD_SPECTR only (else ignored, may be NULL) */
    const float*   draw_uniforms;  /* [B,N] in [0,1): the draw at node n                          */
} mpv_buffers;

#define MPV_COUNTER_NEAR_TIE_ACCEPT 0  /* tests on the accepted walk with |a - u| < 1e-6     */
#define MPV_COUNTER_NEAR_TIE_BONUS  1  /* bonus draws within 1e-6 (relative) of a CDF step   */
#define MPV_COUNTER_ZERO_MASS       2  /* residual updates that found zero mass              */
#define MPV_COUNTER_BAD_TOKEN       3  /* tokens outside [0,V) (treated as never accepted)   */
#define MPV_COUNTER_DEPENDENCY_TIMEOUT 4 /* must stay 0: a node task gave up waiting for its
                                            parent's result (results of that tree are invalid) */
#define MPV_COUNTER_NODE_TASKS_RUN   5  /* (tree, internal node) pairs whose logit rows were
                                          read; the others were proved irrelevant first      */
#define MPV_COUNTER_NODE_TASKS_CANCELLED 6 /* node tasks that had been queued ahead of need and
                                          were dropped unread once their tree was settled     */
#define MPV_COUNTER_NODE_TASKS_RESUMED 7 /* second reads of a row pair: where a tree branches, a
                                          node may first explore its first child's subtree and
                                          come back for the rest only if nothing was accepted  */
#define MPV_COUNTER_COUNT           8  /* length of the counters array        */

/* ABI version of the loaded library (MPV_ABI_VERSION it was built with). */
int mpv_version(void);

/* Static, never-freed description of an error code. */
const char* mpv_strerror(int code);

/* The hipError_t (as int) of the most recent failing HIP call made by this
 * library on the calling thread, 0 if none. */
int mpv_last_hip_error(void);

/* Bytes of device scratch mpv_verify needs for this problem (depends on B, N and
 * the tree only).  Writes *out; returns MPV_OK or an error for an invalid problem. */
int mpv_workspace_bytes(const mpv_problem* problem, size_t* out);

/* Enqueue the whole verification of the batch on `hip_stream` (a hipStream_t
 * passed as void*; NULL = the default stream) and return without waiting.
 * `workspace` is DEVICE memory, 256-byte aligned, of at least
 * mpv_workspace_bytes() bytes, owned by the caller; its contents on entry are
 * ignored and on exit unspecified.  Two calls that share a workspace or output
 * buffers must be ordered by the caller (same stream, or events).
 * The work is done by persistent workgroups grouped in teams; a team takes tasks
 * only once all its workgroups are running, so a call makes progress with whatever
 * share of the device it gets (another kernel, or another call on another stream,
 * may hold compute units).  Every wait inside is bounded (2 s): a launch starved
 * for longer than that gives up and reports it in counters[MPV_COUNTER_DEPENDENCY_TIMEOUT],
 * in which case its outputs are invalid. */
int mpv_verify(const mpv_problem* problem, const mpv_buffers* buffers,
               void* workspace, size_t workspace_bytes, void* hip_stream);

/* mpv_verify for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same operation,
 * arguments, outputs and errors as mpv_verify, with the scratch in a device array of
 * MPV_STATIC_WORKSPACE_BYTES that is part of the library itself (every GPU the library runs on
 * holds its own copy until the process ends).  The call allocates nothing and frees nothing.
 * A problem whose mpv_workspace_bytes() exceeds MPV_STATIC_WORKSPACE_BYTES is refused with
 * MPV_ERR_WORKSPACE before anything is launched (B * N of about 60 000 nodes fits).
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU
 * (different streams, different threads) race and must be ordered by the caller.  The array keeps
 * the previous call's contents; the call itself clears what it needs. */
#define MPV_STATIC_WORKSPACE_BYTES (4u << 20)
int mpv_verify_static(const mpv_problem* problem, const mpv_buffers* buffers, void* hip_stream);

/* Draft trees whose nodes are distinct contexts (Sec. 3, Def. 3.1 and its footnote; Sec. 5, Def. 5.2:
 * paths can overlap after the branching node).  Drafting lays every tree out as `parent` says, each
 * path owning its slots (one row pair, one token, one uniform per slot).  In the tree of Def. 3.1
 * slots drafted for the same context are one node, and the child list of a node keeps one entry per
 * drafted token, in slot order, so it can name the same child several times.
 * mpv_merge_duplicates builds that tree for each of the B token assignments without moving data:
 *   merged_parent[b,n] = the node of the context slot n was drafted after (-1 for n = 0);
 *   context_node[b,n]  = the node of slot n's own context: the first slot (lowest index) drafted for
 *                        it; n itself unless n is a later entry for the same token ("repeat").
 * In merged_parent a repeat has no children (they hang under context_node[b,n] instead), and
 * merged_parent[b,n] < n still holds.  Rows of one context are expected to be equal (the models are
 * functions of the context); only the rows of context nodes matter.
 * parent: HOST [N]; tokens: HOST int32 [B,N] (tokens[b,0] ignored); merged_parent: HOST int32 [B,N],
 * written; context_node: HOST int32 [B,N], written, or NULL.  Host work only: no GPU is touched.
 * Errors: MPV_ERR_NULL, _BAD_SHAPE (B < 0, N < 1), _UNSUPPORTED (N > MPV_MAX_NODES), _BAD_TREE. */
int mpv_merge_duplicates(const int32_t* parent, const int32_t* tokens, int32_t B, int32_t N,
                         int32_t* merged_parent, int32_t* context_node);

/* mpv_verify for a batch in which every tree has a shape of its own: merged_parent is a HOST int32
 * [B,N] array, row b the parent array of tree b (as mpv_merge_duplicates writes it; any valid parent
 * arrays will do).  problem->parent is not read.  Everything else (buffers, layouts, workspace size:
 * what mpv_workspace_bytes gives for a problem of the same B and N, outputs, counters summed over the
 * batch, errors) is as for mpv_verify; path_nodes name context nodes.
 * Why a repeat may be a leaf here: under the SpecInfer solver and under Traversal Verification it is
 * tested only after the first entry for its token was rejected, which leaves that token no residual
 * mass: it is tested with probability 0 and only its residual step remains (App. B, Alg. 4); NSS and
 * Naive move to the first child that carries the drawn token, which is the context node.  SpecTr
 * (App. B, Alg. 3) tests every entry with the entry's own uniform and can accept a repeat; the walk
 * then goes on at the context node.  For that, MPV_METHOD_SPECTR needs context_node: DEVICE int32
 * [B,N], what mpv_merge_duplicates wrote (copied to the device by the caller), borrowed like the
 * buffers; an entry outside [0,N) is ignored (the walk stays at the accepted entry); with the other
 * methods the argument is not read and may be NULL.
 * Cost: the kernels share one shape per launch, so the call makes one mpv_verify launch per run of
 * consecutive trees with equal rows in merged_parent, one after the other on `hip_stream`; lay trees
 * of equal shape next to each other (the shapes are known before the target pass writes its rows).
 * Nothing is launched unless every run is a valid problem. */
int mpv_verify_merged(const mpv_problem* problem, const int32_t* merged_parent, const int32_t* context_node,
                      const mpv_buffers* buffers, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Expected block efficiency of every tree of the batch with the verification's own
 * randomness integrated out (Sec. 5, Eq. 1-3; branching probabilities of Def. 5.3 by
 * the listings of App. D; averaging `expected` over the s trees sampled for one context
 * gives the paper's estimate).  For each tree b:
 *   reach_prob[b,n] = P(node n lies on the accepted path of the rule `problem->method`),
 *                     root: 1  (DEVICE, float32 [B,N]; may be NULL);
 *   expected[b]     = sum_n reach_prob[b,n] = E[tau + 1 | tree b]  (DEVICE, float32 [B]).
 * Top-down rules: the product, along the path, of the probability of moving from a node to
 * the child (an accepted child is moved to itself; a drawn token leads to the first sibling
 * that carries it; SpecInfer tries the children in list order).  Traversal: the nodes are
 * tested in depth-first post-order, each after everything before it was rejected.
 * No uniforms are read and nothing is sampled; every internal node's rows are read once.
 * problem, target_logits, draft_logits, tokens, workspace, hip_stream: as for mpv_verify
 * (same layouts, alignment and workspace size; problem->max_depth is not used beyond its
 * validation).  counters: DEVICE uint32 [MPV_COUNTER_COUNT], zeroed by the call; only
 * ZERO_MASS, BAD_TOKEN, DEPENDENCY_TIMEOUT and NODE_TASKS_RUN are meaningful.
 * Errors: as mpv_verify. */
int mpv_block_efficiency(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                         const int32_t* tokens, void* workspace, size_t workspace_bytes,
                         float* reach_prob, float* expected, uint32_t* counters, void* hip_stream);

/* mpv_block_efficiency for trees of distinct contexts: merged_parent (HOST int32 [B,N], one parent
 * array per tree) and context_node (DEVICE int32 [B,N], read for MPV_METHOD_SPECTR only) as for
 * mpv_verify_merged; problem->parent is not read; one launch per run of consecutive equal rows; the
 * counters are summed.  A later entry for an already drafted token is a leaf of its tree's array:
 * SpecInfer and Traversal never accept it (reach probability 0); under SpecTr its acceptance is
 * credited to the context node, whose reach probability covers every entry that stands for it, and
 * the repeat itself gets 0.  Everything else as for mpv_block_efficiency. */
int mpv_block_efficiency_merged(const mpv_problem* problem, const int32_t* merged_parent, const int32_t* context_node,
                                const void* target_logits, const void* draft_logits, const int32_t* tokens, void* workspace,
                                size_t workspace_bytes, float* reach_prob, float* expected, uint32_t* counters,
                                void* hip_stream);

/* Acceptance rates of the OTLP solver `problem->method` at every internal node of every tree
 * (Sec. 3.2; the listings of App. C): alpha[b,n] = the probability, over k draft tokens drawn
 * i.i.d. from the node's draft distribution (k = the node's number of children in `parent`) and
 * over the solver's own randomness, that the solver's output token is one of the draft tokens.
 * Depends on the node's two logit rows and on k only: no tokens, no uniforms.
 * alpha: DEVICE float32 [B,N]; leaves get 0.  Methods: SPECINFER, NSS, NAIVE, SPECTR;
 * MPV_METHOD_TRAVERSAL returns MPV_ERR_UNSUPPORTED (it is not an OTLP solver; App. C has no rate
 * for it).  Everything else as for mpv_block_efficiency. */
int mpv_acceptance_rates(const mpv_problem* problem, const void* target_logits, const void* draft_logits,
                         void* workspace, size_t workspace_bytes, float* alpha, uint32_t* counters,
                         void* hip_stream);

/* mpv_acceptance_rates for trees of distinct contexts: merged_parent (HOST int32 [B,N], one parent
 * array per tree) as for mpv_verify_merged; problem->parent is not read; one launch per run of
 * consecutive equal rows; the counters are summed.  k of a node is the length of its child list with
 * every entry counted, later entries for an already drafted token included: they are draws from the
 * node's draft distribution like the others (Def. 3.1).  Everything else as for mpv_acceptance_rates. */
int mpv_acceptance_rates_merged(const mpv_problem* problem, const int32_t* merged_parent, const void* target_logits,
                                const void* draft_logits, void* workspace, size_t workspace_bytes, float* alpha,
                                uint32_t* counters, void* hip_stream);

/* Nucleus (top-p) transform of `rows` contiguous logit rows of length V (Sec. 4.1: two of the
 * paper's eight sampling settings use nucleus sampling; the paper does not define it, the usual
 * definition is taken).  With p = softmax(z / T), row by row: the smallest set {v : z_v >= tau},
 * tau one of the row's values, whose mass reaches top_p, is kept; every other token gets the logit
 * -inf, so that verification of the masked rows is verification with the truncated, renormalised
 * distributions.  Tokens with equal logits are kept or dropped together; top_p = 1 keeps every
 * token.  Apply it to the target and to the draft rows (and draw the draft tokens from the
 * masked draft rows) before mpv_verify / mpv_block_efficiency.
 * logits, out: DEVICE, [rows, V] of logit_dtype, 16-byte aligned bases; out may equal logits
 * (in place), otherwise the buffers must not overlap.  Logits must be finite or -inf.
 * threshold_out: DEVICE float32 [rows] or NULL: tau.  kept_out: DEVICE int32 [rows] or NULL: the
 * number of tokens kept.  Errors: MPV_ERR_BAD_SHAPE (rows < 0, V < 1), _UNSUPPORTED (V or rows too
 * large), _BAD_DTYPE, _BAD_TEMPERATURE, _BAD_TOP_P, _NULL, _ALIGNMENT, _HIP. */
int mpv_nucleus_mask(const void* logits, void* out, int32_t logit_dtype, int64_t rows, int32_t V,
                     float temperature, float top_p, float* threshold_out, int32_t* kept_out, void* hip_stream);

/* Softmax statistics of `rows` contiguous logit rows of length V (the first step
 * of the path, exposed on its own): out[r] = { max_v z, ln sum_v exp((z - max)/T) }
 * as float32 pairs.  `logits` and `out` are DEVICE pointers. */
int mpv_row_stats(const void* logits, int32_t logit_dtype, int64_t rows, int32_t V,
                  float temperature, float* out, void* hip_stream);

/* Fill d_u[0..count) (DEVICE) with counter-based uniforms in [0,1): element i is
 * the top 24 bits of the SplitMix64 finaliser applied to
 * seed + (i+1) * 0x9E3779B97F4A7C15, times 2^-24. */
int mpv_fill_uniforms(uint64_t seed, int64_t count, float* d_u, void* hip_stream);

/* Per-launch timing for benchmarks (process-wide state, not thread-safe).
 * mpv_timing_enable(n > 0) creates n pairs of HIP events; from then on every
 * kernel mpv_verify launches carries one pair, which the runtime stamps with the
 * start and the end of that dispatch (nothing extra is put into the caller's
 * stream), until n launches have been recorded.  mpv_timing_enable(0) turns it off
 * and destroys the events.  mpv_timing_read, called after the caller has
 * synchronised that stream, writes the elapsed milliseconds and the MPV_KERNEL_*
 * id of each recorded launch (HOST arrays of `capacity` entries), sets *count and
 * clears the record.  One call is two launches: MPV_KERNEL_INIT (counters, queue) and
 * MPV_KERNEL_NODE_TASK, whose persistent workgroups run every node task (softmax
 * statistics, per-child test probabilities, residual masses) and every sampling task
 * (accept/reject walk, bonus token) of the batch (Sec. 2, step 3); MPV_KERNEL_DEBUG_STATS
 * follows when `stats` is requested. */
#define MPV_KERNEL_INIT        0
#define MPV_KERNEL_NODE_TASK   1
#define MPV_KERNEL_DEBUG_STATS 2
int mpv_timing_enable(int32_t max_launches);
int mpv_timing_read(float* ms_out, int32_t* kernel_out, int32_t capacity, int32_t* count);

#ifdef __cplusplus
}
#endif
#endif /* MPV_H */
