/*
 * libersd -- exponential-race speculative-decoding verification on one AMD MI355X (gfx950).
 *
 * What the entry points compute (paper: Section 3 "Exponential Races"; Algorithm 2 for one drafted
 * token; the sequence extension in Section 3, "an exponential race for every node in the draft
 * sequence"; Algorithm 5 and Section 2 for trees):
 *
 *   For one context, every vocabulary token i gets an exponential e_i ~ Exp(1).  The drafted token is
 *   the race winner under the draft model, argmin_i e_i / Q(i); the token the target model emits is the
 *   winner of the SAME race under the target model, argmin_i e_i / P(i).  A drafted token is accepted
 *   when the two winners agree, and drafted tokens are accepted in order until the first disagreement.
 *
 * With Q = softmax(draft_logits / T), P = softmax(target_logits / T) and the monotone map -log named
 * in Section 3 (Gumbel-max form), argmin_i e_i / p_i = argmax_i ( logit_i / T - ln e_i ): the softmax
 * normaliser does not depend on i and is never computed.
 *
 * Conventions the paper leaves open and this library fixes:
 *   - e_i = -log1p(-v), v = (x + 1/2) * 2^-32, where x is word (i & 3) of
 *     Philox4x32-R( counter = (i >> 2, position-or-node index, sequence index b, draft index d),
 *                   key = (seed & 0xffffffff, seed >> 32) ),  R = ersd_philox_rounds().
 *     The library is built with R = 7, the generator's fastest variant that its authors report as
 *     passing the standard statistical batteries; 10 rounds, their default strength, make the bf16
 *     kernels instruction-bound on this GPU and can be had by compiling with -DERSD_PHILOX_ROUNDS=10.
 *     A caller that decodes several steps passes a fresh seed per step.
 *   - The winner is decided on scores evaluated in IEEE double precision from the exactly widened
 *     logit: score = (double)logit / (double)T - ln e_i.  Exactly equal scores go to the lowest token
 *     index, at every stage of the reduction.
 *   - Position k of a sequence (the extra token emitted after k accepted drafts, Algorithm 2's second
 *     returned token) is drawn by a fresh target-only race on target row k.
 *
 * Memory: all logits, outputs, `parent` and `workspace` are DEVICE pointers owned by the caller.  The
 * library allocates nothing, copies nothing to the host and never synchronises: each call enqueues
 * its kernels on `stream` (a hipStream_t passed as void*, NULL = the default stream) and returns.
 * Outputs are valid once the stream has completed.  Calls are thread safe as long as concurrent
 * calls use distinct workspaces.
 *
 * Layout: tensors are row-major and contiguous with the vocabulary axis innermost; the draft and the
 * target tensor have the same element type.  Logit pointers must be 16-byte aligned, int32 outputs
 * 4-byte aligned, the workspace 16-byte aligned.  V may be any value from 1 to 2^30: rows are streamed with
 * 128-bit loads whatever their alignment (a V that is not a multiple of 8 costs a few percent).
 *
 * Logit contents: -inf is a legal masked token and never wins unless its whole row is -inf, in which
 * case token 0 wins.  Finite logits must satisfy |logit| < 2^100 and |logit| / T < 2^100 (the streaming
 * filter works in fp32, beyond that its products overflow, and it orders bf16 logits by their bit patterns,
 * which holds below 2^121).  NaN and +inf logits, and finite ones beyond those limits, give unspecified
 * tokens (never a fault).
 *
 * Errors: every argument error is detected on the host before any HIP call is made and is returned
 * as a negative status; nothing is enqueued in that case.  ERSD_ERR_HIP reports a failed launch.
 */
#ifndef ERSD_H
#define ERSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ERSD_F32 = 0,  /* IEEE binary32 logits  */
    ERSD_BF16 = 1  /* bfloat16 logits       */
} ersd_dtype;

typedef enum {
    ERSD_OK = 0,
    ERSD_ERR_NULL_POINTER = -1,
    ERSD_ERR_INVALID_ARG = -2,       /* a size < 1, sizes whose products overflow, T not finite or <= 0 */
    ERSD_ERR_UNSUPPORTED_DTYPE = -3,
    ERSD_ERR_MISALIGNED = -4,
    ERSD_ERR_WORKSPACE_TOO_SMALL = -5,
    ERSD_ERR_HIP = -6,
    ERSD_ERR_SCRATCH_TOO_SMALL = -7  /* ersd_race_verify_noalloc: the job needs more than ERSD_NOALLOC_SCRATCH_BYTES */
} ersd_status;

typedef enum { ERSD_VARIANT_SEQUENCE = 0, ERSD_VARIANT_MULTI = 1, ERSD_VARIANT_TREE = 2 } ersd_variant;

/* Scratch memory the library itself holds on every GPU it runs on, for ersd_race_verify_noalloc: 8 MiB. */
#define ERSD_NOALLOC_SCRATCH_BYTES (8u << 20)

/* Arrival trees (Algorithm 5): largest number of arrivals of one race a tree may use, and largest tree. */
#define ERSD_MAX_RANK 8
#define ERSD_MAX_ARRIVAL_TREE_NODES 8192

/*
 * Bytes of device workspace the matching verify call needs (surviving candidates of row segments).
 * `m` is ignored for the sequence and tree variants, `k_or_N` is k (sequence, multi) or N (tree).
 * Returns 0 for invalid sizes.  Pure host computation.
 */
size_t ersd_race_workspace_bytes(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, ersd_dtype dt);

/*
 * Sequence drafting (Section 2 "sequence" strategy verified with the races of Section 3).
 *   draft_logits  [B, k, V]     logits of the draft model at the k drafted positions
 *   target_logits [B, k+1, V]   logits of the target model at those positions plus the bonus position
 *   draft_tokens  [B, k]    out: race winner under the draft model at (b, j)
 *   target_tokens [B, k+1]  out: winner of the same race under the target model; row k is the bonus race
 *   accept_len    [B]       out: number of leading positions j < k with draft_tokens == target_tokens.
 *                           The tokens to emit for sequence b are target_tokens[b, 0 .. accept_len[b]].
 * Race (b, j) uses counter words (i >> 2, j, b, 0).
 */
int ersd_race_verify(const void* draft_logits, const void* target_logits, ersd_dtype dt,
                     int32_t B, int32_t k, int32_t V, float temperature, uint64_t seed,
                     int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * ersd_race_verify for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and kernels, without the
 * workspace: the surviving candidates of the row segments go to a scratch array of ERSD_NOALLOC_SCRATCH_BYTES that
 * the library holds in device memory (one per GPU, from the moment the library is loaded on it until the process
 * ends).  The call allocates nothing and frees nothing.
 *   - A job whose workspace (ersd_race_workspace_bytes) exceeds ERSD_NOALLOC_SCRATCH_BYTES is refused with
 *     ERSD_ERR_SCRATCH_TOO_SMALL; nothing is enqueued.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race on it and give unspecified tokens.  Calls on one stream, or ordered by events, are safe; the
 *     array needs no clearing between calls (every record is written before it is read).
 *   - The first call on a device looks up the array's device address and the kernels' occupancy (queries, no
 *     allocation); ersd_noalloc_prepare does the same ahead of time for the current device, e.g. before a graph
 *     capture begins.  Both return ERSD_ERR_HIP if a query fails.
 */
int ersd_race_verify_noalloc(const void* draft_logits, const void* target_logits, ersd_dtype dt,
                             int32_t B, int32_t k, int32_t V, float temperature, uint64_t seed,
                             int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len, void* stream);
int ersd_noalloc_prepare(void);

/*
 * m independent draft sequences per prompt (a benchmark workload, not a procedure of the paper: the
 * paper's way to use several alternatives at one context is the first arrivals of ONE race, Section 3).
 *   draft_logits [B, m, k, V], target_logits [B, m, k+1, V]
 *   draft_tokens [B, m, k], target_tokens [B, m, k+1], accept_len [B, m] as above per (b, d)
 *   best_len [B]   out: max over d of accept_len[b, d];  best_draft [B] out: lowest d attaining it
 * Race (b, d, j) uses counter words (i >> 2, j, b, d).
 */
int ersd_race_verify_multi(const void* draft_logits, const void* target_logits, ersd_dtype dt,
                           int32_t B, int32_t m, int32_t k, int32_t V, float temperature, uint64_t seed,
                           int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                           int32_t* best_draft, int32_t* best_len,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Draft tree (Section 2 "tree" strategy, walk of Algorithm 5) with one race per node.
 *   draft_logits, target_logits [B, N, V]   per-node logits
 *   parent [N] (device, shared by all B): -1 for children of the token-less root (the prompt context),
 *          otherwise 0 <= parent[n] < n.  Any other value makes node n and its descendants unaccepted.
 *   draft_tokens, target_tokens [B, N]   out: the two winners of race (b, n), counter words (i >> 2, n, b, 0)
 *   accept_len  [B]  out: depth (root children have depth 1) of the deepest node all of whose root path
 *                    agrees; 0 if no root child agrees
 *   accept_node [B]  out, may be NULL: lowest node index attaining accept_len; -1 if accept_len == 0
 * A chain-shaped tree gives the sequence variant's tokens and accept_len (without the bonus race).
 */
int ersd_race_verify_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt,
                          int32_t B, int32_t N, int32_t V, const int32_t* parent,
                          float temperature, uint64_t seed,
                          int32_t* draft_tokens, int32_t* target_tokens,
                          int32_t* accept_len, int32_t* accept_node,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two stages every verify call is made of, for callers that run them apart (a vocabulary-sharded
 * caller gathers the partial winners between them; a profiler times them separately).
 *
 * ersd_race_stage_races runs the races (Section 3) and leaves, in `workspace`, for every race, side and
 * row segment the few tokens that can still be the winner.  ersd_race_stage_accept decides each row's
 * winner among them (in double precision where single precision cannot tell) and runs the acceptance
 * step of the variant (first disagreement, best draft, tree walk).
 * Arguments mean what they mean in the verify call of the same `variant` (ersd_variant; `m` is ignored
 * unless variant is MULTI, k_or_N is k or N); outputs that the variant does not have (best_draft,
 * best_len, accept_node, parent) are ignored and may be NULL.  Both calls must be given the same sizes,
 * element type and workspace; calling them back to back on one stream is exactly the verify call.
 */
int ersd_race_stage_races(int variant, const void* draft_logits, const void* target_logits, ersd_dtype dt,
                          int32_t B, int32_t m, int32_t k_or_N, int32_t V, float temperature, uint64_t seed,
                          void* workspace, size_t workspace_bytes, void* stream);
int ersd_race_stage_accept(int variant, ersd_dtype dt, int32_t B, int32_t m, int32_t k_or_N, int32_t V,
                           float temperature, const int32_t* parent,
                           int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                           int32_t* best_draft, int32_t* best_len, int32_t* accept_node,
                           const void* workspace, size_t workspace_bytes, void* stream);

/*
 * The comparison method on a draft tree: the verification part of Algorithm 4 (Appendix A), recursive rejection over
 * the children of a context, on the layout of ersd_race_verify_arrival_tree (contexts, parent, rank, node validity).
 *   draft_logits, target_logits [B, N + 1, V] (one row per context); draft_tokens [B, N]: what every node drafted
 *   (-1: nothing), e.g. the draft_tokens output of ersd_race_verify_arrival_tree (Algorithm 4 draws the children of
 *   a context from Q without replacement, which the first arrivals of a race under Q are).
 *   plan: the tree's prepared shape (ersd_arrival_tree_prepare on the same parent, rank).
 *   Walk per prompt, from the root context: P_target = P, Q_draft = Q at the context; its valid children are tested
 *   in the order of their ranks: child with token x is accepted iff P_target(x) / Q_draft(x) > U, U = (w + 1/2) 2^-32,
 *   w = word 0 of the Philox counter (rank, context, b, 2), and the walk goes on at the child's context; on a
 *   rejection P_target <- max(P_target - Q_draft, 0) normalised and x leaves Q_draft (normalised again).  When no
 *   child is accepted the step ends with a draw from P_target, made as the race argmin e_i / P_target(i) with e from
 *   the counter (i >> 2, context, b, 1).  A chain with ranks 0 is exactly ersd_gsd_verify.
 *   accept_len [B], accept_node [B] (-1: none), emitted [B, N + 1] out: accepted drafted tokens, the drawn token,
 *   then -1.
 * Precision as for ersd_gsd_verify: probabilities from single-precision exponentials, sums and the residual recursion
 * in double precision; a test whose ratio lies within about 1e-6 (relative) of its uniform, or a draw whose two best
 * scores are as close as the weights' error, may resolve differently from an evaluation in double precision.
 * No workspace; one workgroup per prompt walks its tree; enqueues on `stream`.
 */
int ersd_gsd_verify_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t N,
                         int32_t V, const int32_t* parent, const int32_t* rank, const void* plan, size_t plan_bytes,
                         const int32_t* draft_tokens, float temperature, uint64_t seed,
                         int32_t* accept_len, int32_t* accept_node, int32_t* emitted, void* stream);

/*
 * Host-only description of how a job is cut into shares of equal cost for `blocks` workgroups (1..4096): every
 * row is a run of 8-token groups, rows are laid end to end, and share b covers the global group indices
 * [block_start[b], block_start[b+1]).  The cost of a share is 10 per group of a row pair, 5 per group of a
 * target-only row, plus *out_seg_cost for every row whose first group it holds.  A row's partial winners are
 * written by the workgroups row_first[r] .. row_last[r], one slot each, at most *out_nslot of them.
 *   out_G, out_nslot: never NULL.  out_seg_cost: may be NULL.  block_start: NULL or [G + 1] (G <= blocks).
 *   row_first, row_last: both NULL or both [rows], rows = B * m * (k + 1) or B * N.  All HOST arrays.  No device
 *   work is done.
 */
int ersd_plan_describe_host(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, ersd_dtype dt,
                            uint32_t blocks, uint32_t* out_G, uint32_t* out_nslot, uint32_t* out_seg_cost,
                            uint64_t* block_start, uint32_t* row_first, uint32_t* row_last);

/*
 * The same for an arrival tree (ersd_race_verify_arrival_tree), whose partition depends on which contexts have
 * children: need_host[N + 1] (HOST) holds, per context, the number of arrivals its children ask for (0: no child, the
 * context's draft row is not read), as the library derives it on the device from (parent, rank).  Rows are the
 * B * (N + 1) contexts; a context with a draft row costs 10 per group, one without 5.
 */
int ersd_arrival_plan_describe_host(int32_t B, int32_t N, int32_t V, ersd_dtype dt, const int32_t* need_host,
                                    uint32_t blocks, uint32_t* out_G, uint32_t* out_nslot, uint64_t* block_start,
                                    uint32_t* row_first, uint32_t* row_last);

/*
 * Test and tuning hooks: not part of the product interface.  Process-wide settings that the tests use to reach
 * code paths a default launch does not take (a row cut into many segments, the exhaustive scoring path).  A
 * field at its default leaves the library's own choice in place; NULL restores all defaults.
 * Set them while no call of this library is running, and keep them unchanged between the two stage calls of one
 * job and between a workspace-size query and the call it serves.
 */
typedef struct {
    int32_t force_blocks;      /* > 0: workgroups the race kernels are launched with (default 0: as many as are resident) */
    int32_t exhaustive;        /* != 0: every token is scored in double precision inside the race kernels (default 0) */
    int32_t seg_cost_units;    /* >= 0: cost charged to every row start when the job is cut up (default -1) */
    int32_t align_groups;      /* >= 0: 8-token groups a share's start is aligned to, a power of two; 0 or 1: none (default -1) */
} ersd_test_hooks;
void ersd_test_hooks_set(const ersd_test_hooks* hooks);

/*
 * The race of ONE model's logits, for callers that draft and verify at different times (the order of
 * Algorithm 2: the draft model's race picks the drafted token, the target model is evaluated on it, and
 * only then is the same race run under the target model).  Because the exponentials are a function of
 * (seed, sequence, draft, position, token) alone, racing the draft rows and the target rows in separate
 * calls gives exactly the tokens of the fused verify calls.
 *   logits [B, m, npos, V]: rows of one model at positions pos0 .. pos0 + npos - 1 of every sequence
 *   tokens [B, m, npos] out: race winner of row (b, d, j), counter words (i >> 2, pos0 + j, b, d)
 * A drafting loop calls it with npos = 1 and pos0 = the step; verification calls it on the target
 * logits with pos0 = 0, npos = k + 1 (sequence, multi) or npos = N (tree: positions are node indices).
 * Workspace size: ersd_race_sample_workspace_bytes.  Same memory, stream and error rules as above.
 */
int ersd_race_sample(const void* logits, ersd_dtype dt, int32_t B, int32_t m, int32_t npos, int32_t V,
                     int32_t pos0, float temperature, uint64_t seed, int32_t* tokens,
                     void* workspace, size_t workspace_bytes, void* stream);
size_t ersd_race_sample_workspace_bytes(int32_t B, int32_t m, int32_t npos, int32_t V, ersd_dtype dt);

/*
 * The acceptance step alone, on tokens the caller already holds (device arrays laid out as in the verify
 * call of the same `variant`): first disagreement per draft (Section 2), best draft, or the tree walk.
 * Outputs the variant does not have are ignored and may be NULL.
 */
int ersd_accept_lengths(int variant, int32_t B, int32_t m, int32_t k_or_N, const int32_t* parent,
                        const int32_t* draft_tokens, const int32_t* target_tokens, int32_t* accept_len,
                        int32_t* best_draft, int32_t* best_len, int32_t* accept_node, void* stream);

/*
 * Tree verification as Algorithm 5 states it (Section 3: the batch strategy takes the first arrivals of ONE
 * race under the draft model as the alternatives at a context; the tree strategy continues each of them).
 * This is the form for which the emitted tokens keep the target model's distribution.
 *   Contexts: c = 0 is the partial output, c = n + 1 the path that ends at node n; C = N + 1.  Context c has
 *   one race, counter words (i >> 2, c, b, 0).
 *   draft_logits, target_logits [B, C, V]; draft row (b, c) is read only if context c has a valid child.
 *   parent, rank [N] (DEVICE, shared by all prompts): node n is the child of context parent[n] + 1 that holds
 *   arrival number rank[n] (0 = the winner) of that context's race under the draft model.  Arrivals are ordered
 *   by decreasing score logit/T - ln e, equal scores by increasing token index; a token whose score is -inf
 *   never arrives, and a missing arrival is token -1.  Node n is valid iff -1 <= parent[n] < n, its parent is
 *   valid, 0 <= rank[n] < ERSD_MAX_RANK and no earlier valid sibling has the same rank; an invalid node gets
 *   draft token -1 and is never accepted.  N <= ERSD_MAX_ARRIVAL_TREE_NODES.
 *   draft_tokens [B, N] out: the token each node drafts.  target_tokens [B, C] out: the winner of each
 *   context's race under the target model.
 *   Walk (the listing's second loop, with the race under the target model as its comment says, continuing at
 *   the matching child): at the current context emit the target winner; if a valid child drafted that token,
 *   accept it and go on at that child's context, else stop.
 *   accept_len [B] out: accepted drafted tokens.  accept_node [B] out: last accepted node, -1 if none.
 *   emitted [B, C] out: the accept_len + 1 tokens the step produces (accepted tokens, then the correction or
 *   bonus token), then -1.
 * A chain with all ranks 0 gives exactly ersd_race_verify (draft rows 0 .. N-1, target rows 0 .. N).
 * Workspace size: ersd_race_arrival_tree_workspace_bytes (0 for invalid sizes).  Same memory, stream and
 * error rules as ersd_race_verify; the tree is examined on the device, nothing is read back.
 */
int ersd_race_verify_arrival_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt,
                                  int32_t B, int32_t N, int32_t V, const int32_t* parent, const int32_t* rank,
                                  float temperature, uint64_t seed,
                                  int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                                  int32_t* accept_node, int32_t* emitted,
                                  void* workspace, size_t workspace_bytes, void* stream);
size_t ersd_race_arrival_tree_workspace_bytes(int32_t B, int32_t N, int32_t V, ersd_dtype dt);

/*
 * The same with the tree's shape derived ahead of time.  A drafting tree is built once and verified against many
 * steps (Section 4: the optimal tree depends on the acceptance function, not on the step); what the library derives
 * from (parent, rank) alone, which nodes are valid, how many arrivals every context must deliver, what every
 * context costs, takes one small kernel that ersd_race_verify_arrival_tree runs on every call.
 *   ersd_arrival_tree_prepare writes that into `plan` (DEVICE memory of the caller, 16-byte aligned, at least
 *   ersd_arrival_tree_plan_bytes(N) bytes; enqueued on `stream`).
 *   ersd_race_verify_arrival_tree_prepared is ersd_race_verify_arrival_tree with row strides (elements between row
 *   starts, >= V) that reads the plan instead: same arguments otherwise, same results.  The plan must have been
 *   prepared from the same (parent, rank) and be complete on `stream`'s timeline; it is only read and may serve any
 *   number of calls, also concurrent ones.
 */
size_t ersd_arrival_tree_plan_bytes(int32_t N);
int ersd_arrival_tree_prepare(const int32_t* parent, const int32_t* rank, int32_t N, void* plan, size_t plan_bytes,
                              void* stream);
int ersd_race_verify_arrival_tree_prepared(const void* draft_logits, int64_t draft_row_stride,
                                           const void* target_logits, int64_t target_row_stride, ersd_dtype dt,
                                           int32_t B, int32_t N, int32_t V, const int32_t* parent, const int32_t* rank,
                                           const void* plan, size_t plan_bytes, float temperature, uint64_t seed,
                                           int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                                           int32_t* accept_node, int32_t* emitted,
                                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same calls for logits whose rows do not lie back to back: a head that pads the vocabulary, or a slice
 * [..., :V] of a wider tensor.  Row r of a tensor (r counts its leading axes in row-major order: (b, j),
 * (b, d, j), (b, n) or (b, c)) starts `row_stride` ELEMENTS after row r - 1; each row is V contiguous
 * elements.  row_stride >= V (else ERSD_ERR_INVALID_ARG); the two tensors may have different strides.  The
 * base pointers must be 16-byte aligned as before, the rows themselves need element alignment only.
 * Results, workspace sizes, stream and error rules are those of the call without `_strided`, which is the
 * case row_stride == V.
 */
int ersd_race_verify_strided(const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                             int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t k, int32_t V,
                             float temperature, uint64_t seed, int32_t* draft_tokens, int32_t* target_tokens,
                             int32_t* accept_len, void* workspace, size_t workspace_bytes, void* stream);
int ersd_race_verify_multi_strided(const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                                   int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t m, int32_t k,
                                   int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens,
                                   int32_t* target_tokens, int32_t* accept_len, int32_t* best_draft,
                                   int32_t* best_len, void* workspace, size_t workspace_bytes, void* stream);
int ersd_race_verify_tree_strided(const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                                  int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t N, int32_t V,
                                  const int32_t* parent, float temperature, uint64_t seed, int32_t* draft_tokens,
                                  int32_t* target_tokens, int32_t* accept_len, int32_t* accept_node,
                                  void* workspace, size_t workspace_bytes, void* stream);
int ersd_race_sample_strided(const void* logits, int64_t row_stride, ersd_dtype dt, int32_t B, int32_t m,
                             int32_t npos, int32_t V, int32_t pos0, float temperature, uint64_t seed,
                             int32_t* tokens, void* workspace, size_t workspace_bytes, void* stream);
int ersd_race_verify_arrival_tree_strided(const void* draft_logits, int64_t draft_row_stride,
                                          const void* target_logits, int64_t target_row_stride, ersd_dtype dt,
                                          int32_t B, int32_t N, int32_t V, const int32_t* parent,
                                          const int32_t* rank, float temperature, uint64_t seed,
                                          int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                                          int32_t* accept_node, int32_t* emitted, void* workspace,
                                          size_t workspace_bytes, void* stream);

/* Host helper: 1 if every node of (parent, rank)[0..N) (HOST arrays) is valid by the rule above, else 0. */
int ersd_arrival_tree_validate_host(const int32_t* parent_host, const int32_t* rank_host, int32_t N);

/*
 * Optimal drafting tree, Algorithm 3 (Section 4), for a 0-th order acceptance function as in the paper's
 * experiments (Section 5): R(j_1 .. j_l) = r[j_1] * ... * r[j_l], r[j] = accept_by_rank[j] = probability that the
 * child holding arrival j of a context is accepted given that its parent was.  Greedy growth from a priority
 * queue, O(k log k).  All pointers are HOST arrays; no device work.
 *   accept_by_rank [nr]: values in [0, 1] that do not increase with j (a later arrival is accepted less often;
 *   the algorithm offers sibling j + 1 only after sibling j was taken); nr = largest number of children of a vertex
 *   (<= ERSD_MAX_RANK for use with ersd_race_verify_arrival_tree).
 *   parent, rank [k] out: the k vertices with the largest R, in the order they were taken (so parent[n] < n; -1 =
 *   the root), in the layout ersd_race_verify_arrival_tree takes.  Equal acceptance values are taken by depth,
 *   then by index tuple, so the result is a function of the arguments alone.
 *   node_accept [k] out or NULL: R of every vertex.  expected_accepted out or NULL: their sum, the expected
 *   number of accepted drafted tokens under the model.
 * Returns ERSD_OK, ERSD_ERR_NULL_POINTER, or ERSD_ERR_INVALID_ARG (nr < 1, k < 1, a value outside [0, 1] or larger
 * than its predecessor).
 */
int ersd_tree_build_optimal_host(const double* accept_by_rank, int32_t nr, int32_t k, int32_t* parent,
                                 int32_t* rank, double* node_accept, double* expected_accepted);

/*
 * The fixed tree of the SpecInfer kind used as a comparison strategy in Section 5: `branches` sequences that share
 * their first `shared` drafted tokens (the paper: 3 sequences, 2 common tokens).  The prefix is a chain of winners;
 * the branches leave it as arrivals 0 .. branches-1 of the prefix's last context and continue as chains of
 * winners, growing in turn until k vertices are placed.  parent, rank [k] out (HOST).
 */
int ersd_tree_build_specinfer_host(int32_t k, int32_t shared, int32_t branches, int32_t* parent, int32_t* rank);

/*
 * Verification by the comparison method, GSD (Section 2; Algorithm 1 applied position by position, as the text
 * on the sequence strategy says), on the same kind of inputs as ersd_race_verify: it is here so that the cost of
 * the two methods can be measured side by side.
 *   draft_logits [B, k, V], target_logits [B, k + 1, V], draft_tokens [B, k] (DEVICE; the tokens the drafting
 *   stage drew from Q = softmax(draft / T); ersd_race_sample is one way to draw them; a value outside [0, V) is
 *   rejected at its position without being used as an index).
 *   Position j of sequence b accepts its drafted token x iff P(x) / Q(x) > U, U = (w + 1/2) 2^-32 with w = word 0
 *   of the Philox counter (0, j, b, 2).  accept_len [B] out: tokens accepted before the first rejection, a.
 *   next_token [B] out: for a < k a draw from the residual max(P - Q, 0) / sum at position a, for a == k a draw
 *   from P at position k; both by an exponential race (argmin e_i / weight_i, e from the counter (i >> 2, a, b, 1),
 *   lowest index on ties); a row whose weights are all zero gives token 0.
 * The normalisers are accumulated in single precision, so an acceptance test whose ratio lies within about 1e-6
 * (relative) of its uniform, or a residual whose two best scores are closer than what an error of 1e-6 (p + q) in
 * the weights can move them, may resolve differently from an evaluation in double precision.
 * Workspace size: ersd_gsd_workspace_bytes (0 for invalid sizes).  Same memory, stream and error rules as
 * ersd_race_verify.
 */
int ersd_gsd_verify(const void* draft_logits, const void* target_logits, ersd_dtype dt,
                    int32_t B, int32_t k, int32_t V, const int32_t* draft_tokens,
                    float temperature, uint64_t seed, int32_t* accept_len, int32_t* next_token,
                    void* workspace, size_t workspace_bytes, void* stream);
size_t ersd_gsd_workspace_bytes(int32_t B, int32_t k, int32_t V, ersd_dtype dt);

/* ERSD_MAX_RANK of the loaded library. */
int ersd_max_rank(void);

/*
 * Device self-check of the facts the streaming filter relies on.  The two single-precision bounds, over all 2^32
 * generator words, against double precision; and the packed half-precision maximum used as an order on bf16 bit
 * patterns, over all pairs of in-domain patterns.  counters: DEVICE array of 5 uint64, written as
 *   [0] words whose cheap upper bound of -log2 e fell below the true value      (must be 0)
 *   [1] words whose refined log2 e is off by more than 2^-9                    (must be 0)
 *   [2] largest refinement error, [3] largest upper-bound slack (IEEE fp32 bit patterns)
 *   [4] bf16 pairs whose packed maximum fell below the larger value             (must be 0)
 * Enqueues on `stream`; takes a fraction of a second.
 */
int ersd_selftest_bounds(uint64_t* counters, void* stream);

/*
 * Measurement aid: reads the device buffers a and b (b may be NULL with b_bytes 0) exactly once with the race
 * kernel's load instructions and launch shape and does nothing else, so that a benchmark can print what the memory
 * system gives a kernel of this shape beside the race kernel's own rate.  Sizes are multiples of 16 bytes, the
 * buffers 16-byte aligned; sink is a DEVICE uint32 that is practically never written.  Enqueues on `stream`.
 */
int ersd_read_probe(const void* a, size_t a_bytes, const void* b, size_t b_bytes, void* sink, void* stream);

/* Host helper: 1 if parent[0..N) (a HOST array) satisfies the tree contract above, else 0. */
int ersd_tree_validate_host(const int32_t* parent_host, int32_t N);

/* Static text for a status code (never NULL). */
const char* ersd_status_string(int status);

/* Rounds of the Philox4x32 generator this library was compiled with (7 unless rebuilt). */
int ersd_philox_rounds(void);

/* major * 10000 + minor * 100 + patch */
int ersd_version(void);

#ifdef __cplusplus
}
#endif
#endif
