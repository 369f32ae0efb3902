/*
 * CPU oracle for exponential-race speculative-decoding verification (ERSD).
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain, fp64 definition of what
 * the GPU library must compute.  It shares no code with the HIP path and is
 * never linked into it; only the tests, the smoke check and the CPU-baseline
 * leg of the benchmark may call it.
 *
 * All pointers are HOST pointers owned by the caller.  Logit tensors are
 * row-major with the vocabulary innermost; dtype 0 = IEEE fp32, dtype 1 =
 * bfloat16 (upper 16 bits of an fp32, widened exactly).
 *
 * What is computed (paper: Section 3 "Exponential Races", Algorithm 2 for
 * k = 1, the sequence extension of Section 3, Algorithm 5 for trees):
 *   one race per context: e_i ~ Exp(1) for every token i, the draft token is
 *   argmin_i e_i / Q(i), the target token is argmin_i e_i / P(i) with the SAME
 *   e; a drafted token is accepted while the two winners agree.
 * With P = softmax(l_p / T), Q = softmax(l_q / T) and the monotone map -log
 * (Section 3 calls this the Gumbel-max form) argmin e_i/p_i equals
 * argmax_i ( l_i / T - ln e_i ), because the softmax normaliser does not
 * depend on i.
 *
 * Readings the paper leaves open (RNG, bit layout, tie-break, temperature):
 *   e_i = -log1p(-v),  v = (x + 1/2) * 2^-32,  x = word (i & 3) of
 *   Philox4x32-R( counter = (i >> 2, position-or-node, sequence, draft),
 *                 key = (seed low word, seed high word) ),  R = 7 by default;
 *   exact score ties go to the lowest token index.
 */
#ifndef ERSD_ORACLE_H
#define ERSD_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Philox4x32 with `rounds` rounds (Salmon, Moraes, Dror, Shaw 2011). */
void oracle_philox4x32(int rounds, const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Number of Philox rounds used by every race below (default 7, the round count the GPU library is built with;
 * 10 is the generator's standard strength and the one its published known answers are for). */
void oracle_set_rounds(int rounds);
int oracle_get_rounds(void);

/* Exp(1) variate and its Gumbel -ln(e) from one 32-bit word. */
double oracle_exponential(uint32_t x);
double oracle_gumbel(uint32_t x);

/* Per-row diagnostics, one entry per logit row that was raced. */
typedef struct {
    int32_t token;      /* lowest index attaining the maximum score            */
    int32_t runner_up;  /* index of the best score among the other tokens, -1 if V == 1 */
    double s1;          /* winning score  l/T - ln e  (natural-log units)      */
    double s2;          /* runner-up score (-inf if V == 1)                    */
    int32_t near_tie;   /* 1 iff s1 - s2 <= 1e-6 * max(1, |s1|) (or s1 == s2)  */
    int32_t exact_tie;  /* 1 iff s1 == s2                                      */
} oracle_row_info;

/*
 * One race over up to two rows that share the same exponentials.
 * rows[s] may be NULL for an absent side.  c1, c2, c3 are counter words 1..3.
 */
void oracle_race_rows(const void* const rows[2], int dtype, int64_t V, float temperature,
                      uint64_t seed, uint32_t c1, uint32_t c2, uint32_t c3,
                      oracle_row_info info[2]);

/* Tokens whose score is within tol_rel * max(1,|s1|) of the row maximum, in
 * increasing index order; returns how many exist (writes at most cap). */
int64_t oracle_row_candidates(const void* row, int dtype, int64_t V, float temperature,
                              uint64_t seed, uint32_t c1, uint32_t c2, uint32_t c3,
                              double tol_rel, int32_t* out_idx, int64_t cap);

/*
 * One model's races: logits [B,m,npos,V] at positions pos0 .. pos0+npos-1, tokens [B,m,npos]; race (b,d,j)
 * uses counter words (i >> 2, pos0 + j, b, d), i.e. the exponentials of the two-model race at that place
 * (Algorithm 2 runs the draft race first and the target race, on the same e, after the target evaluation).
 */
int oracle_race_sample(const void* logits, int dtype, int32_t B, int32_t m, int32_t npos, int64_t V, int32_t pos0,
                       float temperature, uint64_t seed, int32_t* tokens, oracle_row_info* info);

/*
 * Sequence variant.  draft [B,k,V], target [B,k+1,V].
 * draft_tokens [B,k], target_tokens [B,k+1], accept_len [B];
 * draft_info [B,k] and target_info [B,k+1] may be NULL.
 * Returns 0, or -1 on invalid arguments.
 */
int oracle_race_verify(const void* draft, const void* target, int dtype,
                       int32_t B, int32_t k, int64_t V, float temperature, uint64_t seed,
                       int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                       oracle_row_info* draft_info, oracle_row_info* target_info);

/*
 * Multi-draft variant (workload definition, not a procedure of the paper):
 * draft [B,m,k,V], target [B,m,k+1,V]; counter word 3 is the draft index.
 * accept_len [B,m]; best_len[b] = max over drafts, best_draft[b] = lowest
 * draft index attaining it.
 */
int oracle_race_verify_multi(const void* draft, const void* target, int dtype,
                             int32_t B, int32_t m, int32_t k, int64_t V,
                             float temperature, uint64_t seed,
                             int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                             int32_t* best_draft, int32_t* best_len,
                             oracle_row_info* draft_info, oracle_row_info* target_info);

/*
 * Tree variant: one race per node (counter word 1 = node index), draft and
 * target [B,N,V], parent[N] shared by all sequences with parent[n] == -1 for
 * children of the (token-less) root and 0 <= parent[n] < n otherwise; any
 * other value makes node n (and its descendants) unaccepted.
 * accept_len[b] = depth of the deepest node whose whole root path agrees
 * (0 if none), accept_node[b] = lowest such node index (-1 if none).
 */
int oracle_race_verify_tree(const void* draft, const void* target, int dtype,
                            int32_t B, int32_t N, int64_t V, const int32_t* parent,
                            float temperature, uint64_t seed,
                            int32_t* draft_tokens, int32_t* target_tokens,
                            int32_t* accept_len, int32_t* accept_node,
                            oracle_row_info* draft_info, oracle_row_info* target_info);

/*
 * Tree form as Algorithm 5 states it (Section 3: the batch strategy takes the first arrivals of ONE race under Q
 * as the alternatives at a context, and the tree strategy continues each of them).
 *   Contexts: c = 0 is the partial output, c = n + 1 the path that ends at node n; C = N + 1.  Context c has one
 *   race, counter words (i >> 2, c, b, 0).  draft and target are [B,C,V]; draft row (b,c) is read only if c has a
 *   child.  Node n is the child of context parent[n] + 1 that holds arrival number rank[n] (0 = the winner) of that
 *   context's race under Q: tokens ordered by decreasing score l_q/T - ln e, equal scores by increasing index;
 *   a token whose score is -inf (outside the support) never arrives, and a missing arrival is token -1.
 *   Node n is valid iff -1 <= parent[n] < n, the parent is valid, 0 <= rank[n] < max_rank and no earlier valid
 *   sibling has the same rank; an invalid node has draft token -1 and is never accepted.
 *   Walk (the listing's second loop, reading its race as the one under P, as its comment says, and moving on to the
 *   matching child): at the current context emit the winner under P; if a valid child drafted that token, accept
 *   it and continue at the child's context, else stop.
 * Outputs: arrivals [B,C,max_rank] (the first need[c] arrivals, -1 elsewhere), draft_tokens [B,N],
 * target_tokens [B,C], accept_len [B] = accepted drafted tokens, accept_node [B] = last accepted node (-1 if none),
 * emitted [B,C] = the accept_len + 1 tokens the step produces, then -1.
 * arrival_near_tie [B,C] (may be NULL): 1 iff two consecutive arrivals among the first need[c] + 1 are closer than
 * 1e-6 * max(1, |score|).  target_info [B,C] may be NULL.
 */
int oracle_race_verify_arrival_tree(const void* draft, const void* target, int dtype, int32_t B, int32_t N, int64_t V,
                                    const int32_t* parent, const int32_t* rank, int32_t max_rank,
                                    float temperature, uint64_t seed,
                                    int32_t* arrivals, int32_t* draft_tokens, int32_t* target_tokens,
                                    int32_t* accept_len, int32_t* accept_node, int32_t* emitted,
                                    int32_t* arrival_near_tie, oracle_row_info* target_info);

/* valid[N] and need[N+1] (arrivals wanted per context) of a (parent, rank) tree, by the rule above. */
void oracle_arrival_tree_shape(const int32_t* parent, const int32_t* rank, int32_t N, int32_t max_rank,
                               int32_t* valid, int32_t* need);

/*
 * GSD, the comparison method (Section 2; Algorithm 1 applied position by position, as the prose on the sequence
 * strategy says: drafted tokens are verified in order until the first rejection).
 *   draft [B,k,V], target [B,k+1,V], draft_tokens [B,k]: the tokens the drafting stage sampled from Q.
 *   Position j of sequence b: P = softmax(l_p / T), Q = softmax(l_q / T); the drafted token x is accepted iff
 *   P(x) / Q(x) > U with U = (w + 1/2) 2^-32, w = word 0 of the Philox counter (0, j, b, 2).
 *   accept_len[b] = a = number of accepted tokens.  next_token[b]: if a < k a draw from the residual
 *   max(P - Q, 0) / sum at position a, if a == k a draw from P at position k; both by an exponential race
 *   argmin e_i / weight_i with e from the counter (i >> 2, a, b, 1) (the appendix notes that GSD's draws can be
 *   made with races; any sampler would do).  A row whose weights are all zero gives token 0.
 * The results above are exact in double precision and carry no tolerance.  info[b] (may be NULL) reports how
 * sensitive they are, for a caller that compares an implementation with inexact normalisers against this one and
 * says how inexact: min_accept_gap = smallest |ratio - U| / max(ratio, U) over the tested positions; near_accept =
 * 1 iff that is <= accept_rel_tol; rivals = number of other tokens that could win the final race if every weight
 * moved by weight_rel_tol (p + q); lse_p, lse_q: normalisers at the last tested position.  With both tolerances 0
 * the flags report exact coincidences only.
 */
typedef struct {
    int32_t near_accept;
    int32_t rivals;
    double lse_p, lse_q;
    double score; /* winning score ln(weight) - ln(e) of the final race */
    double min_accept_gap;
} oracle_gsd_info;

int oracle_gsd_verify(const void* draft, const void* target, int dtype, int32_t B, int32_t k, int64_t V,
                      const int32_t* draft_tokens, float temperature, uint64_t seed,
                      int32_t* accept_len, int32_t* next_token, oracle_gsd_info* info, double accept_rel_tol,
                      double weight_rel_tol);
double oracle_logsumexp(const void* row, int dtype, int64_t V, float temperature);
double oracle_gsd_uniform(uint64_t seed, uint32_t j, uint32_t b);
double oracle_gsd_uniform_ctr(uint64_t seed, uint32_t r, uint32_t j, uint32_t b);

/*
 * GSD on a draft tree: the verification part of Algorithm 4 (Appendix A), recursive rejection over the children of
 * a context.  Tree layout, contexts and node validity as in oracle_race_verify_arrival_tree; draft, target [B,N+1,V];
 * draft_tokens [B,N]: what every node drafted (-1: nothing), given by the caller (Algorithm 4 draws the children of
 * a context from Q without replacement, i.e. the first arrivals of a race under Q).
 *   At a context: P_target = P, Q_draft = Q; its valid children are tested in the order of their ranks; child with
 *   token x is accepted iff P_target(x) / Q_draft(x) > U, U = (w + 1/2) 2^-32 with w = word 0 of the counter
 *   (rank, context, b, 2), and the walk goes on at the child's context with fresh distributions; on a rejection
 *   P_target <- max(P_target - Q_draft, 0) normalised, Q_draft(x) <- 0 and normalised.  When no child is accepted
 *   the step ends with a draw from P_target by the race argmin e_i / P_target(i), e from (i >> 2, context, b, 1).
 *   A distribution that becomes all zero stays so (no further acceptance; the draw gives token 0).
 * accept_len [B], accept_node [B] (-1: none), emitted [B,N+1]: accepted drafted tokens, the drawn token, then -1.
 * info, accept_rel_tol, weight_rel_tol: the sensitivity report of oracle_gsd_verify (rivals here: other tokens that
 * could win the draw if every weight moved by weight_rel_tol of itself).  A chain with ranks 0 equals
 * oracle_gsd_verify on the same rows.
 */
int oracle_gsd_verify_tree(const void* draft, const void* target, int dtype, int32_t B, int32_t N, int64_t V,
                           const int32_t* parent, const int32_t* rank, int32_t max_rank, const int32_t* draft_tokens,
                           float temperature, uint64_t seed, int32_t* accept_len, int32_t* accept_node,
                           int32_t* emitted, oracle_gsd_info* info, double accept_rel_tol, double weight_rel_tol);

/* Threads the row loops will use (OpenMP), for reporting. */
int oracle_num_threads(void);
void oracle_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
