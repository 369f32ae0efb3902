/*
 * CPU oracle for exponential-race speculative-decoding verification.
 * TEST INFRASTRUCTURE ONLY -- see ersd_oracle.h.  Plain C, fp64, one pass per
 * row, no blocking or fusion beyond sharing one exponential between the draft
 * and the target row of a race (which is the method: Section 3 uses the same
 * realisation of e for P and Q).
 */
#include "ersd_oracle.h"

#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef ORACLE_PHILOX_ROUNDS
#define ORACLE_PHILOX_ROUNDS 7
#endif
static int g_rounds = ORACLE_PHILOX_ROUNDS;
static int g_threads = 0; /* 0 = OpenMP default */

void oracle_set_rounds(int rounds) { g_rounds = rounds; }
int oracle_get_rounds(void) { return g_rounds; }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}
void oracle_set_num_threads(int n) { g_threads = n; }

/* ---- Philox4x32 (Salmon et al. 2011): two 32x32->64 multiplies per round ---- */
void oracle_philox4x32(int rounds, const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < rounds; ++r) {
        if (r > 0) { /* Weyl key schedule between rounds */
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ---- e ~ Exp(1) from a 32-bit word: v uniform on the 2^32 midpoints of (0,1) ---- */
double oracle_exponential(uint32_t x) {
    double v = ((double)x + 0.5) * (1.0 / 4294967296.0);
    return -log1p(-v);
}

/* Section 3: arrival times map to Gumbel noise through the monotone -log. */
double oracle_gumbel(uint32_t x) { return -log(oracle_exponential(x)); }

static double widen(const void* row, int dtype, int64_t i) {
    if (dtype == 0) {
        return (double)((const float*)row)[i];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t*)row)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

static void finish_info(oracle_row_info* r) {
    r->exact_tie = 0;
    r->near_tie = 0;
    if (r->runner_up < 0) return;
    if (r->s1 == r->s2) { /* also covers -inf == -inf */
        r->exact_tie = 1;
        r->near_tie = 1;
        return;
    }
    double scale = fabs(r->s1) > 1.0 ? fabs(r->s1) : 1.0;
    if (r->s1 - r->s2 <= 1e-6 * scale) r->near_tie = 1;
}

void oracle_race_rows(const void* const rows[2], int dtype, int64_t V, float temperature,
                      uint64_t seed, uint32_t c1, uint32_t c2, uint32_t c3,
                      oracle_row_info info[2]) {
    const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    const double T = (double)temperature;
    for (int s = 0; s < 2; ++s) {
        info[s].token = -1;
        info[s].runner_up = -1;
        info[s].s1 = -INFINITY;
        info[s].s2 = -INFINITY;
        info[s].near_tie = 0;
        info[s].exact_tie = 0;
    }
    uint32_t words[4] = {0, 0, 0, 0};
    for (int64_t i = 0; i < V; ++i) {
        if ((i & 3) == 0) {
            const uint32_t ctr[4] = {(uint32_t)(i >> 2), c1, c2, c3};
            oracle_philox4x32(g_rounds, ctr, key, words);
        }
        const double g = oracle_gumbel(words[i & 3]); /* -ln e_i, shared by both sides */
        for (int s = 0; s < 2; ++s) {
            if (!rows[s]) continue;
            /* argmin e_i / p_i  ==  argmax  l_i/T - ln e_i  (normaliser dropped) */
            const double score = widen(rows[s], dtype, i) / T + g;
            oracle_row_info* r = &info[s];
            if (r->token < 0) { /* first token */
                r->token = (int32_t)i;
                r->s1 = score;
            } else if (score > r->s1) { /* strictly better: new winner, old winner becomes runner-up */
                r->runner_up = r->token;
                r->s2 = r->s1;
                r->token = (int32_t)i;
                r->s1 = score;
            } else if (r->runner_up < 0 || score > r->s2) { /* ties keep the lower index */
                r->runner_up = (int32_t)i;
                r->s2 = score;
            }
        }
    }
    for (int s = 0; s < 2; ++s)
        if (rows[s]) finish_info(&info[s]);
}

int64_t oracle_row_candidates(const void* row, int dtype, int64_t V, float temperature,
                              uint64_t seed, uint32_t c1, uint32_t c2, uint32_t c3,
                              double tol_rel, int32_t* out_idx, int64_t cap) {
    const void* rows[2] = {row, NULL};
    oracle_row_info info[2];
    oracle_race_rows(rows, dtype, V, temperature, seed, c1, c2, c3, info);
    const double s1 = info[0].s1;
    const double scale = fabs(s1) > 1.0 ? fabs(s1) : 1.0;
    const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    const double T = (double)temperature;
    uint32_t words[4] = {0, 0, 0, 0};
    int64_t n = 0;
    for (int64_t i = 0; i < V; ++i) {
        if ((i & 3) == 0) {
            const uint32_t ctr[4] = {(uint32_t)(i >> 2), c1, c2, c3};
            oracle_philox4x32(g_rounds, ctr, key, words);
        }
        const double score = widen(row, dtype, i) / T + oracle_gumbel(words[i & 3]);
        if (score == s1 || s1 - score <= tol_rel * scale) {
            if (n < cap) out_idx[n] = (int32_t)i;
            ++n;
        }
    }
    return n;
}

static size_t elem_size(int dtype) { return dtype == 0 ? 4 : 2; }

static int bad_common(const void* draft, const void* target, int dtype, int64_t V, float T) {
    if (!draft || !target) return 1;
    if (dtype != 0 && dtype != 1) return 1;
    if (V < 1 || V > 2147483647LL) return 1;
    if (!(T > 0.0f) || !isfinite(T)) return 1;
    return 0;
}

/* Leading positions where the draft and target winners agree (Section 2:
 * drafted tokens are accepted in order until the first rejection). */
static int32_t accepted_prefix(const int32_t* d, const int32_t* t, int32_t k) {
    int32_t a = 0;
    while (a < k && d[a] == t[a]) ++a;
    return a;
}

int oracle_race_verify_multi(const void* draft, const void* target, int dtype,
                             int32_t B, int32_t m, int32_t k, int64_t V,
                             float temperature, uint64_t seed,
                             int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                             int32_t* best_draft, int32_t* best_len,
                             oracle_row_info* draft_info, oracle_row_info* target_info) {
    if (bad_common(draft, target, dtype, V, temperature)) return -1;
    if (B < 1 || m < 1 || k < 1 || !draft_tokens || !target_tokens || !accept_len) return -1;
    const size_t es = elem_size(dtype);
    const int64_t nrace = (int64_t)B * m * (k + 1);
    if (g_threads > 0) {
#ifdef _OPENMP
        omp_set_num_threads(g_threads);
#endif
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrace; ++r) {
        const int32_t j = (int32_t)(r % (k + 1));
        const int32_t d = (int32_t)((r / (k + 1)) % m);
        const int32_t b = (int32_t)(r / ((int64_t)(k + 1) * m));
        const int64_t seq = (int64_t)b * m + d;
        /* position k is the bonus position: a target-only race (Algorithm 2's
         * extra token after an accepted draft, drawn here by a fresh race). */
        const char* drow = j < k ? (const char*)draft + (size_t)((seq * k + j) * V) * es : NULL;
        const char* trow = (const char*)target + (size_t)((seq * (k + 1) + j) * V) * es;
        const void* rows[2] = {drow, trow};
        oracle_row_info info[2];
        oracle_race_rows(rows, dtype, V, temperature, seed, (uint32_t)j, (uint32_t)b, (uint32_t)d, info);
        if (j < k) {
            draft_tokens[seq * k + j] = info[0].token;
            if (draft_info) draft_info[seq * k + j] = info[0];
        }
        target_tokens[seq * (k + 1) + j] = info[1].token;
        if (target_info) target_info[seq * (k + 1) + j] = info[1];
    }
    for (int64_t seq = 0; seq < (int64_t)B * m; ++seq)
        accept_len[seq] = accepted_prefix(draft_tokens + seq * k, target_tokens + seq * (k + 1), k);
    if (best_draft && best_len) {
        for (int32_t b = 0; b < B; ++b) {
            int32_t bl = -1, bd = -1;
            for (int32_t d = 0; d < m; ++d) {
                if (accept_len[(int64_t)b * m + d] > bl) {
                    bl = accept_len[(int64_t)b * m + d];
                    bd = d;
                }
            }
            best_len[b] = bl;
            best_draft[b] = bd;
        }
    }
    return 0;
}

int oracle_race_sample(const void* logits, int dtype, int32_t B, int32_t m, int32_t npos, int64_t V, int32_t pos0,
                       float temperature, uint64_t seed, int32_t* tokens, oracle_row_info* info) {
    if (bad_common(logits, logits, dtype, V, temperature)) return -1;
    if (B < 1 || m < 1 || npos < 1 || pos0 < 0 || !tokens) return -1;
    const size_t es = elem_size(dtype);
    const int64_t nrace = (int64_t)B * m * npos;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrace; ++r) {
        const int32_t j = (int32_t)(r % npos);
        const int32_t d = (int32_t)((r / npos) % m);
        const int32_t b = (int32_t)(r / ((int64_t)npos * m));
        /* a one-model race: the same counters as the two-model race at that (sequence, draft, position) */
        const void* rows[2] = {NULL, (const char*)logits + (size_t)(r * V) * es};
        oracle_row_info out[2];
        oracle_race_rows(rows, dtype, V, temperature, seed, (uint32_t)(pos0 + j), (uint32_t)b, (uint32_t)d, out);
        tokens[r] = out[1].token;
        if (info) info[r] = out[1];
    }
    return 0;
}

int oracle_race_verify(const void* draft, const void* target, int dtype,
                       int32_t B, int32_t k, int64_t V, float temperature, uint64_t seed,
                       int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                       oracle_row_info* draft_info, oracle_row_info* target_info) {
    /* the sequence variant is the multi-draft layout with one draft (counter word 3 = 0) */
    return oracle_race_verify_multi(draft, target, dtype, B, 1, k, V, temperature, seed,
                                    draft_tokens, target_tokens, accept_len, NULL, NULL,
                                    draft_info, target_info);
}

int oracle_race_verify_tree(const void* draft, const void* target, int dtype,
                            int32_t B, int32_t N, int64_t V, const int32_t* parent,
                            float temperature, uint64_t seed,
                            int32_t* draft_tokens, int32_t* target_tokens,
                            int32_t* accept_len, int32_t* accept_node,
                            oracle_row_info* draft_info, oracle_row_info* target_info) {
    if (bad_common(draft, target, dtype, V, temperature)) return -1;
    if (B < 1 || N < 1 || !parent || !draft_tokens || !target_tokens || !accept_len) return -1;
    const size_t es = elem_size(dtype);
    const int64_t nrace = (int64_t)B * N;
    if (g_threads > 0) {
#ifdef _OPENMP
        omp_set_num_threads(g_threads);
#endif
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrace; ++r) {
        const int32_t n = (int32_t)(r % N);
        const int32_t b = (int32_t)(r / N);
        const void* rows[2] = {(const char*)draft + (size_t)(r * V) * es,
                               (const char*)target + (size_t)(r * V) * es};
        oracle_row_info info[2];
        oracle_race_rows(rows, dtype, V, temperature, seed, (uint32_t)n, (uint32_t)b, 0u, info);
        draft_tokens[r] = info[0].token;
        target_tokens[r] = info[1].token;
        if (draft_info) draft_info[r] = info[0];
        if (target_info) target_info[r] = info[1];
    }
    /* A node is accepted iff the two winners agree at it and at every ancestor
     * (Section 4: a vertex can only be accepted if its ancestors are). */
    for (int32_t b = 0; b < B; ++b) {
        int32_t best_depth = 0, best_node = -1;
        for (int32_t n = 0; n < N; ++n) {
            int32_t depth = 0, ok = 1, cur = n, steps = 0;
            while (1) {
                if (draft_tokens[(int64_t)b * N + cur] != target_tokens[(int64_t)b * N + cur]) { ok = 0; break; }
                ++depth;
                const int32_t p = parent[cur];
                if (p == -1) break;
                if (p < 0 || p >= cur || ++steps > N) { ok = 0; break; } /* malformed tree */
                cur = p;
            }
            if (ok && depth > best_depth) {
                best_depth = depth;
                best_node = n;
            }
        }
        accept_len[b] = best_depth;
        if (accept_node) accept_node[b] = best_node;
    }
    return 0;
}

/* ---- Algorithm 5 as printed: one race per context, the children of a context are its first arrivals under Q ---- */

void oracle_arrival_tree_shape(const int32_t* parent, const int32_t* rank, int32_t N, int32_t max_rank,
                               int32_t* valid, int32_t* need) {
    for (int32_t c = 0; c <= N; ++c) need[c] = 0;
    for (int32_t n = 0; n < N; ++n) {
        const int32_t p = parent[n], r = rank[n];
        int ok = p >= -1 && p < n && r >= 0 && r < max_rank && (p == -1 || valid[p]);
        for (int32_t o = 0; ok && o < n; ++o) /* an earlier sibling already holds this arrival */
            if (valid[o] && parent[o] == p && rank[o] == r) ok = 0;
        valid[n] = ok;
        if (ok && r + 1 > need[p + 1]) need[p + 1] = r + 1;
    }
}

/* position of (score a, index ia) after (score b, index ib) in the order of arrival: earlier arrival = larger score,
 * equal scores in index order */
static int arrives_after(double a, int64_t ia, double b, int64_t ib) { return a < b || (a == b && ia > ib); }

int oracle_race_verify_arrival_tree(const void* draft, const void* target, int dtype, int32_t B, int32_t N, int64_t V,
                                    const int32_t* parent, const int32_t* rank, int32_t max_rank,
                                    float temperature, uint64_t seed,
                                    int32_t* arrivals, int32_t* draft_tokens, int32_t* target_tokens,
                                    int32_t* accept_len, int32_t* accept_node, int32_t* emitted,
                                    int32_t* arrival_near_tie, oracle_row_info* target_info) {
    if (bad_common(draft, target, dtype, V, temperature)) return -1;
    if (B < 1 || N < 1 || max_rank < 1 || !parent || !rank || !arrivals || !draft_tokens || !target_tokens ||
        !accept_len || !accept_node || !emitted)
        return -1;
    const size_t es = elem_size(dtype);
    const int32_t C = N + 1; /* contexts: 0 = the partial output itself, n + 1 = the path that ends at node n */
    int32_t* valid = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int32_t* need = (int32_t*)malloc(sizeof(int32_t) * (size_t)C);
    if (!valid || !need) { free(valid); free(need); return -1; }
    oracle_arrival_tree_shape(parent, rank, N, max_rank, valid, need);
    const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    const double T = (double)temperature;
    const int64_t nrace = (int64_t)B * C;
    if (g_threads > 0) {
#ifdef _OPENMP
        omp_set_num_threads(g_threads);
#endif
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrace; ++r) {
        const int32_t c = (int32_t)(r % C);
        const int32_t b = (int32_t)(r / C);
        /* winner under P of the race of context c */
        const void* rows[2] = {NULL, (const char*)target + (size_t)(r * V) * es};
        oracle_row_info info[2];
        oracle_race_rows(rows, dtype, V, temperature, seed, (uint32_t)c, (uint32_t)b, 0u, info);
        target_tokens[r] = info[1].token;
        if (target_info) target_info[r] = info[1];
        for (int32_t a = 0; a < max_rank; ++a) arrivals[r * max_rank + a] = -1;
        if (arrival_near_tie) arrival_near_tie[r] = 0;
        if (need[c] == 0) continue; /* no child: Q is not evaluated at this context */
        /* the same race under Q: every token's score, then the first need[c] arrivals one after the other */
        const char* qrow = (const char*)draft + (size_t)(r * V) * es;
        double* s = (double*)malloc(sizeof(double) * (size_t)V);
        if (!s) { failed = 1; continue; }
        uint32_t words[4] = {0, 0, 0, 0};
        for (int64_t i = 0; i < V; ++i) {
            if ((i & 3) == 0) {
                const uint32_t ctr[4] = {(uint32_t)(i >> 2), (uint32_t)c, (uint32_t)b, 0u};
                oracle_philox4x32(g_rounds, ctr, key, words);
            }
            s[i] = widen(qrow, dtype, i) / T + oracle_gumbel(words[i & 3]);
        }
        double ps = INFINITY;
        int64_t pi = -1;
        for (int32_t a = 0; a <= need[c]; ++a) { /* one more than needed, to see how close the next one was */
            int64_t bi = -1;
            for (int64_t i = 0; i < V; ++i) {
                if (!(s[i] > -INFINITY)) continue; /* a token outside the support never arrives */
                if (a > 0 && !arrives_after(s[i], i, ps, pi)) continue;
                if (bi < 0 || s[i] > s[bi]) bi = i;
            }
            if (bi < 0) break;
            if (a > 0 && arrival_near_tie) {
                const double scale = fabs(ps) > 1.0 ? fabs(ps) : 1.0;
                if (ps == s[bi] || ps - s[bi] <= 1e-6 * scale) arrival_near_tie[r] = 1;
            }
            if (a < need[c]) arrivals[r * max_rank + a] = (int32_t)bi;
            ps = s[bi];
            pi = bi;
        }
        free(s);
    }
    if (failed) { free(valid); free(need); return -1; }
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t n = 0; n < N; ++n)
            draft_tokens[(int64_t)b * N + n] =
                valid[n] ? arrivals[((int64_t)b * C + parent[n] + 1) * max_rank + rank[n]] : -1;
        /* verification walk: emit the winner under P; go on from the child that drafted it, if there is one */
        for (int32_t c = 0; c < C; ++c) emitted[(int64_t)b * C + c] = -1;
        int32_t ctx = 0, len = 0, node = -1;
        while (1) {
            const int32_t t = target_tokens[(int64_t)b * C + ctx];
            emitted[(int64_t)b * C + len] = t;
            int32_t next = -1;
            for (int32_t n = 0; n < N && next < 0; ++n)
                if (valid[n] && parent[n] + 1 == ctx && draft_tokens[(int64_t)b * N + n] == t) next = n;
            if (next < 0) break;
            ++len;
            node = next;
            ctx = next + 1;
        }
        accept_len[b] = len;
        accept_node[b] = node;
    }
    free(valid);
    free(need);
    return 0;
}

/* ---- GSD (Section 2, Algorithm 1 applied position by position): the comparison method ---- */

/* log sum_i exp(l_i / T) of one row, two plain passes (maximum, then sum). -inf for a row without support. */
double oracle_logsumexp(const void* row, int dtype, int64_t V, float temperature) {
    const double T = (double)temperature;
    double m = -INFINITY;
    for (int64_t i = 0; i < V; ++i) {
        const double z = widen(row, dtype, i) / T;
        if (z > m) m = z;
    }
    if (!(m > -INFINITY) || m == INFINITY) return m;
    double sum = 0.0;
    for (int64_t i = 0; i < V; ++i) sum += exp(widen(row, dtype, i) / T - m);
    return m + log(sum);
}

/* the uniform of the acceptance test at (sequence b, position j): word 0 of the counter (0, j, b, 2) */
/* the uniform of an acceptance test: word 0 of the counter (r, j, b, 2); r = 0 in the sequence form, the child's
 * rank in the tree form */
double oracle_gsd_uniform_ctr(uint64_t seed, uint32_t r, uint32_t j, uint32_t b) {
    const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    const uint32_t ctr[4] = {r, j, b, 2u};
    uint32_t w[4];
    oracle_philox4x32(g_rounds, ctr, key, w);
    return ((double)w[0] + 0.5) * (1.0 / 4294967296.0);
}
double oracle_gsd_uniform(uint64_t seed, uint32_t j, uint32_t b) { return oracle_gsd_uniform_ctr(seed, 0u, j, b); }

int oracle_gsd_verify(const void* draft, const void* target, int dtype, int32_t B, int32_t k, int64_t V,
                      const int32_t* draft_tokens, float temperature, uint64_t seed,
                      int32_t* accept_len, int32_t* next_token, oracle_gsd_info* info, double accept_rel_tol,
                      double weight_rel_tol) {
    if (bad_common(draft, target, dtype, V, temperature)) return -1;
    if (B < 1 || k < 1 || !draft_tokens || !accept_len || !next_token) return -1;
    for (int64_t t = 0; t < (int64_t)B * k; ++t)
        if (draft_tokens[t] < 0 || draft_tokens[t] >= V) return -1;
    const size_t es = elem_size(dtype);
    const double T = (double)temperature;
    const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    if (g_threads > 0) {
#ifdef _OPENMP
        omp_set_num_threads(g_threads);
#endif
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        /* verification: drafted tokens are tested in order until the first rejection */
        int32_t a = 0;
        int near_accept = 0;
        double min_gap = INFINITY;
        double lse_p = 0.0, lse_q = 0.0;
        for (; a < k; ++a) {
            const char* qrow = (const char*)draft + (size_t)(((int64_t)b * k + a) * V) * es;
            const char* prow = (const char*)target + (size_t)(((int64_t)b * (k + 1) + a) * V) * es;
            lse_q = oracle_logsumexp(qrow, dtype, V, temperature);
            lse_p = oracle_logsumexp(prow, dtype, V, temperature);
            const int32_t x = draft_tokens[(int64_t)b * k + a];
            /* P(x) / Q(x) > U */
            const double ratio = exp((widen(prow, dtype, x) / T - lse_p) - (widen(qrow, dtype, x) / T - lse_q));
            const double U = oracle_gsd_uniform(seed, (uint32_t)a, (uint32_t)b);
            const double big = ratio > U ? ratio : U;
            const double gap = fabs(ratio - U) / big;
            if (gap < min_gap) min_gap = gap;
            if (gap <= accept_rel_tol) near_accept = 1;
            if (!(ratio > U)) break;
        }
        accept_len[b] = a;
        /* next token: from the residual max(P - Q, 0) at the rejected position, or from P after the last draft;
         * both drawn by an exponential race with the counter (i >> 2, a, b, 1) */
        const char* prow = (const char*)target + (size_t)(((int64_t)b * (k + 1) + a) * V) * es;
        const char* qrow = a < k ? (const char*)draft + (size_t)(((int64_t)b * k + a) * V) * es : NULL;
        if (a == k) lse_p = oracle_logsumexp(prow, dtype, V, temperature);
        int64_t best = -1;
        double s1 = -INFINITY, floor1 = -INFINITY;
        uint32_t words[4] = {0, 0, 0, 0};
        for (int64_t i = 0; i < V; ++i) {
            if ((i & 3) == 0) {
                const uint32_t ctr[4] = {(uint32_t)(i >> 2), (uint32_t)a, (uint32_t)b, 1u};
                oracle_philox4x32(g_rounds, ctr, key, words);
            }
            const double p = exp(widen(prow, dtype, i) / T - lse_p);
            const double q = qrow ? exp(widen(qrow, dtype, i) / T - lse_q) : 0.0;
            const double w = p - q > 0.0 ? p - q : 0.0;
            const double score = log(w) + oracle_gumbel(words[i & 3]); /* argmin e_i / w_i */
            if (best < 0 || score > s1) {
                best = i;
                s1 = score;
                const double wl = w - weight_rel_tol * (p + q);
                floor1 = wl > 0.0 ? log(wl) + oracle_gumbel(words[i & 3]) : -INFINITY;
            }
        }
        next_token[b] = s1 > -INFINITY ? (int32_t)best : 0;
        if (info) {
            /* how many other tokens could win if every weight moved by weight_rel_tol (p + q): the sensitivity of
             * the residual to relative errors of the two normalisers, for whoever compares an implementation
             * with inexact normalisers against this one */
            int32_t rivals = 0;
            for (int64_t i = 0; i < V; ++i) {
                if ((i & 3) == 0) {
                    const uint32_t ctr[4] = {(uint32_t)(i >> 2), (uint32_t)a, (uint32_t)b, 1u};
                    oracle_philox4x32(g_rounds, ctr, key, words);
                }
                if (i == best) continue;
                const double p = exp(widen(prow, dtype, i) / T - lse_p);
                const double q = qrow ? exp(widen(qrow, dtype, i) / T - lse_q) : 0.0;
                const double w = p - q > 0.0 ? p - q : 0.0;
                const double top = log(w + weight_rel_tol * (p + q)) + oracle_gumbel(words[i & 3]);
                if (top >= floor1) ++rivals;
            }
            info[b].near_accept = near_accept;
            info[b].min_accept_gap = min_gap;
            info[b].rivals = rivals;
            info[b].lse_p = lse_p;
            info[b].lse_q = a < k ? lse_q : 0.0;
            info[b].score = s1;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------------------------------
 * GSD on a draft tree (Algorithm 4, verification part; recursive rejection over the children of a context).
 * The drafted tokens are given (Algorithm 4 draws the children of a context from Q without replacement, which is
 * what the first arrivals of a race under Q are; the caller supplies them).  Per prompt, from the root context:
 *   P_target <- P(. | context), Q_draft <- Q(. | context)
 *   for the valid children of the context in the order of their ranks (a child whose drafted token is -1, a missing
 *   arrival, is passed over): accept the child if P_target(x) / Q_draft(x) > U, U from the counter
 *   (rank, context, b, 2), and go on at the child's context with fresh distributions; else
 *       P_target <- max(P_target - Q_draft, 0); P_target <- P_target / sum(P_target)
 *       Q_draft(x) <- 0;                        Q_draft  <- Q_draft / sum(Q_draft)
 *   when no child is accepted (or there is none) the step ends with a draw from P_target, made as an exponential
 *   race argmin e_i / P_target(i) with e from the counter (i >> 2, context, b, 1).
 * A distribution that becomes all zero stays all zero (then nothing more is accepted and the draw gives token 0).
 * accept_len[b], accept_node[b] (-1: none), emitted[b][C]: the accepted drafted tokens, then the drawn token, then -1.
 * info (may be NULL) as for oracle_gsd_verify, over all tested children and the final draw; the two tolerances only
 * shape that report.  A chain with ranks 0 gives exactly oracle_gsd_verify.
 */
int oracle_gsd_verify_tree(const void* draft, const void* target, int dtype, int32_t B, int32_t N, int64_t V,
                           const int32_t* parent, const int32_t* rank, int32_t max_rank, const int32_t* draft_tokens,
                           float temperature, uint64_t seed, int32_t* accept_len, int32_t* accept_node,
                           int32_t* emitted, oracle_gsd_info* info, double accept_rel_tol, double weight_rel_tol) {
    if (bad_common(draft, target, dtype, V, temperature)) return -1;
    if (B < 1 || N < 1 || max_rank < 1 || !parent || !rank || !draft_tokens || !accept_len || !accept_node || !emitted)
        return -1;
    for (int64_t t = 0; t < (int64_t)B * N; ++t)
        if (draft_tokens[t] < -1 || draft_tokens[t] >= V) return -1;
    const int32_t C = N + 1;
    int32_t* valid = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    int32_t* need = (int32_t*)malloc(sizeof(int32_t) * (size_t)C);
    if (!valid || !need) { free(valid); free(need); return -1; }
    oracle_arrival_tree_shape(parent, rank, N, max_rank, valid, need);
    const size_t es = elem_size(dtype);
    const double T = (double)temperature;
    const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    if (g_threads > 0) {
#ifdef _OPENMP
        omp_set_num_threads(g_threads);
#endif
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        double* P = (double*)malloc(sizeof(double) * (size_t)V);
        double* Q = (double*)malloc(sizeof(double) * (size_t)V);
        if (!P || !Q) { free(P); free(Q); failed = 1; continue; }
        int32_t ctx = 0, len = 0, node = -1, near_accept = 0;
        double min_gap = INFINITY, lse_p = 0.0, lse_q = 0.0;
        int32_t* out = emitted + (int64_t)b * C;
        for (int32_t c = 0; c < C; ++c) out[c] = -1;
        for (;;) {
            const char* prow = (const char*)target + (size_t)(((int64_t)b * C + ctx) * V) * es;
            const char* qrow = (const char*)draft + (size_t)(((int64_t)b * C + ctx) * V) * es;
            lse_p = oracle_logsumexp(prow, dtype, V, temperature);
            for (int64_t i = 0; i < V; ++i) P[i] = exp(widen(prow, dtype, i) / T - lse_p);
            int32_t accepted = -1;
            if (need[ctx] > 0) {
                lse_q = oracle_logsumexp(qrow, dtype, V, temperature);
                for (int64_t i = 0; i < V; ++i) Q[i] = exp(widen(qrow, dtype, i) / T - lse_q);
                for (int32_t r = 0; r < max_rank && accepted < 0; ++r) {
                    int32_t child = -1; /* the valid child of this context that holds arrival r */
                    for (int32_t n = 0; n < N; ++n)
                        if (valid[n] && parent[n] + 1 == ctx && rank[n] == r) { child = n; break; }
                    if (child < 0) continue;
                    const int32_t x = draft_tokens[(int64_t)b * N + child];
                    if (x < 0) continue;
                    const double ratio = P[x] / Q[x]; /* Q[x] > 0 for a token that was drawn from Q */
                    const double U = oracle_gsd_uniform_ctr(seed, (uint32_t)r, (uint32_t)ctx, (uint32_t)b);
                    const double big = ratio > U ? ratio : U;
                    const double gap = fabs(ratio - U) / big;
                    if (gap < min_gap) min_gap = gap;
                    if (gap <= accept_rel_tol) near_accept = 1;
                    if (ratio > U) { accepted = child; break; }
                    double sp = 0.0, sq = 0.0;
                    for (int64_t i = 0; i < V; ++i) { P[i] = P[i] - Q[i] > 0.0 ? P[i] - Q[i] : 0.0; sp += P[i]; }
                    if (sp > 0.0) for (int64_t i = 0; i < V; ++i) P[i] /= sp;
                    Q[x] = 0.0;
                    for (int64_t i = 0; i < V; ++i) sq += Q[i];
                    if (sq > 0.0) for (int64_t i = 0; i < V; ++i) Q[i] /= sq;
                }
            }
            if (accepted >= 0) {
                out[len++] = draft_tokens[(int64_t)b * N + accepted];
                node = accepted;
                ctx = accepted + 1;
                continue;
            }
            /* the draw from what is left of P at this context */
            int64_t best = -1;
            double s1 = -INFINITY, floor1 = -INFINITY;
            uint32_t words[4] = {0, 0, 0, 0};
            for (int64_t i = 0; i < V; ++i) {
                if ((i & 3) == 0) {
                    const uint32_t ctr[4] = {(uint32_t)(i >> 2), (uint32_t)ctx, (uint32_t)b, 1u};
                    oracle_philox4x32(g_rounds, ctr, key, words);
                }
                const double score = log(P[i]) + oracle_gumbel(words[i & 3]);
                if (best < 0 || score > s1) {
                    best = i;
                    s1 = score;
                    const double wl = P[i] * (1.0 - weight_rel_tol);
                    floor1 = wl > 0.0 ? log(wl) + oracle_gumbel(words[i & 3]) : -INFINITY;
                }
            }
            out[len] = s1 > -INFINITY ? (int32_t)best : 0;
            if (info) {
                int32_t rivals = 0;
                for (int64_t i = 0; i < V; ++i) {
                    if ((i & 3) == 0) {
                        const uint32_t ctr[4] = {(uint32_t)(i >> 2), (uint32_t)ctx, (uint32_t)b, 1u};
                        oracle_philox4x32(g_rounds, ctr, key, words);
                    }
                    if (i == best) continue;
                    if (log(P[i] * (1.0 + weight_rel_tol)) + oracle_gumbel(words[i & 3]) >= floor1) ++rivals;
                }
                info[b].near_accept = near_accept;
                info[b].min_accept_gap = min_gap;
                info[b].rivals = rivals;
                info[b].lse_p = lse_p;
                info[b].lse_q = lse_q;
                info[b].score = s1;
            }
            break;
        }
        accept_len[b] = len;
        accept_node[b] = node;
        free(P);
        free(Q);
    }
    free(valid);
    free(need);
    return failed ? -1 : 0;
}
