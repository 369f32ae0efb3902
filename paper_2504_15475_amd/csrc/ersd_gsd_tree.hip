// libersd: GSD on a draft tree, the verification part of Algorithm 4 of the paper (Appendix A; recursive rejection
// over the children of a context), for gfx950.  The comparison method's counterpart of the arrival-tree verification:
// on the same logits and the same drafted tokens it shows what the paper's remark on simplicity means in kernel
// terms.  Where the race needs one pass over each row and decides every context at once, this walk is sequential
// per prompt: it needs the two normalisers of a context before its first test, a further pass over both rows for
// every rejected child (the normaliser of the residual max(P - Q, 0)), and a last pass for the draw, and it cannot
// start on a context before the walk has reached it.
//
// One workgroup per prompt walks the tree.  Per context:
//   normalisers : maximum and sum of 2^(z - max) over the target row (and the draft row if the context has children),
//                 z = logit * log2(e) / T; single-precision terms, double-precision sums.
//   children    : in the order of their ranks; P_target(x) / Q_draft(x) > U with U from the counter
//                 (rank, context, b, 2).  After j rejections the two distributions are functions of the token's own
//                 two probabilities, the rejected tokens and j + 1 scalars, so nothing is stored per token:
//                     Q_j(t) = Q(t) [t not rejected] / S_j,          S_j = 1 - sum of Q over the rejected tokens
//                     P_j(t) = max(P_{j-1}(t) - Q_{j-1}(t), 0) / Z_j, Z_j = sum over t of the numerator
//                 and a rejection costs one pass over both rows for the next Z.
//   draw        : a race over the weights P_j(t), counter (i >> 2, context, b, 1): single-precision scores with a
//                 margin find the few tokens that can win, which are rescored with the exact exponential.
// The rows of one context (at most 2 MB) stay in the L2 cache between the passes.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "ersd.h"
#include "ersd_philox.h"
#include "ersd_tree_plan.h"

namespace {

using ersd_philox::philox4x32;

constexpr int kThreads = 1024;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr int kListCap = 1024;
constexpr int kMaxRank = ERSD_MAX_RANK;
constexpr float kNone = -3.0e38f;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float widen(const char* row, int dt, int32_t i) {
    if (dt == ERSD_F32) return reinterpret_cast<const float*>(row)[i];
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(row)[i] << 16);
}

// four consecutive logits (i a multiple of 4): one 8- or 16-byte load when the row allows it
template <bool VEC>
__device__ __forceinline__ void load4(const char* row, int dt, int32_t i, int32_t V, float out[4]) {
    if (VEC) {
        if (dt == ERSD_F32) {
            const u32x4 r = *reinterpret_cast<const u32x4*>(row + (size_t)i * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = __uint_as_float(r[e]);
        } else {
            const u32x2 r = *reinterpret_cast<const u32x2*>(row + (size_t)i * 2);
            out[0] = __uint_as_float(r[0] << 16); out[1] = __uint_as_float(r[0] & 0xffff0000u);
            out[2] = __uint_as_float(r[1] << 16); out[3] = __uint_as_float(r[1] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = i + e < V ? widen(row, dt, i + e) : -INFINITY;
    }
}

// log2 of e = -ln(1 - v), v = (x + 1/2) 2^-32, in single precision; |error| < 2^-7
__device__ __forceinline__ float log2_exponential(uint32_t x) {
    if (x < (1u << 23)) {
        const float v = ((float)x + 0.5f) * 0x1p-32f;
        const float poly = fmaf(v, fmaf(v, fmaf(v, fmaf(v, 0.2f, 0.25f), 0.33333334f), 0.5f), 1.0f);
        return __builtin_amdgcn_logf(v * poly);
    }
    const float y = (float)(~x) + 0.5f;
    const float e2 = 32.0f - __builtin_amdgcn_logf(y);
    return __builtin_amdgcn_logf(e2) - 0.5287663729f;
}
constexpr float kLogErr = 0x1p-5f + 0x1p-10f;  // log2_exponential (2^-7), v_log_f32, and the final subtraction

struct TreeArgs {
    const char* draft;
    const char* target;
    const int32_t* parent;
    const int32_t* rank;
    const int32_t* valid;         // from the prepared tree shape
    const int32_t* draft_tokens;  // [B, N]
    int32_t* accept_len;
    int32_t* accept_node;
    int32_t* emitted;             // [B, C]
    int32_t B, N, V;
    int dt;
    float c2;                     // log2(e) / T
    double c2d;
    uint32_t key0, key1;
};

// What the walk knows at a context after some rejections: wavefront-uniform, kept in LDS.
struct State {
    double lse2_p, lse2_q;        // normalisers in log2 units
    double S[kMaxRank + 1];       // Q mass left after j rejections (S[0] = 1)
    double Z[kMaxRank + 1];       // Z[j]: normaliser of the residual after j rejections (Z[0] unused)
    int32_t removed[kMaxRank];    // rejected tokens, in order
    int32_t nrej;
    int32_t dead;                 // a residual summed to zero: nothing is left of P
};

__device__ __forceinline__ double block_sum(double v, double* red) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    __syncthreads();  // red may still be read from the previous reduction
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < kWaves; ++w) s += red[w];  // every thread adds in the same order
    return s;
}
__device__ __forceinline__ float block_max(float v, double* red) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = (double)v;
    __syncthreads();
    float m = kNone;
    for (int w = 0; w < kWaves; ++w) m = fmaxf(m, (float)red[w]);
    return m;
}

// P_j(t) of a token from its own two probabilities: the recursion of the residuals, in double precision.
// `q0` is the token's probability under Q (0 if the context's Q was not evaluated).
__device__ __forceinline__ double residual_weight(const State& st, int32_t t, double p0, double q0, int32_t level) {
    double P = p0;
    bool gone = false;  // rejected at an earlier level: no longer in Q_draft
    for (int32_t i = 0; i < level; ++i) {
        const double Qi = gone ? 0.0 : q0 / st.S[i];
        const double d = P - Qi;
        P = d > 0.0 ? d / st.Z[i + 1] : 0.0;
        gone = gone || st.removed[i] == t;
    }
    return P;
}

template <bool VEC>
__device__ void walk_prompt(const TreeArgs& a, int32_t b) {
    const int tid = threadIdx.x;
    const int32_t N = a.N, C = N + 1, V = a.V;
    const int es = a.dt == ERSD_F32 ? 4 : 2;
    __shared__ State st;
    __shared__ double red[kWaves];
    __shared__ int32_t child_of_rank[kMaxRank];
    __shared__ int32_t decision;  // node accepted at this context, or -1
    __shared__ int32_t count;
    __shared__ int32_t cand[kListCap];
    __shared__ uint32_t cword[kListCap];
    __shared__ double best_s[kWaves];
    __shared__ int32_t best_i[kWaves];

    int32_t* out = a.emitted + (int64_t)b * C;
    for (int32_t c = tid; c < C; c += kThreads) out[c] = -1;
    int32_t ctx = 0, len = 0, node = -1;
    const int32_t ngroups = (V + 3) >> 2;

    while (true) {  // one context per trip; the context index grows with every trip, so at most C trips
        const char* prow = a.target + (size_t)((int64_t)b * C + ctx) * V * es;
        const char* qrow = a.draft + (size_t)((int64_t)b * C + ctx) * V * es;
        // the valid children of this context, by rank
        if (tid < kMaxRank) child_of_rank[tid] = -1;
        __syncthreads();
        for (int32_t n = tid; n < N; n += kThreads)
            if (a.valid[n] && a.parent[n] + 1 == ctx) child_of_rank[a.rank[n]] = n;  // ranks of valid siblings differ
        __syncthreads();
        bool has_children = false;
        for (int r = 0; r < kMaxRank; ++r) has_children = has_children || child_of_rank[r] >= 0;

        // normalisers: maxima, then sums
        float mp = kNone, mq = kNone;
        for (int32_t g = tid; g < ngroups; g += kThreads) {
            float lp[4], lq[4];
            load4<VEC>(prow, a.dt, g * 4, V, lp);
#pragma unroll
            for (int e = 0; e < 4; ++e) mp = fmaxf(mp, lp[e] * a.c2);
            if (has_children) {
                load4<VEC>(qrow, a.dt, g * 4, V, lq);
#pragma unroll
                for (int e = 0; e < 4; ++e) mq = fmaxf(mq, lq[e] * a.c2);
            }
        }
        mp = block_max(mp, red);
        mq = has_children ? block_max(mq, red) : 0.0f;
        double sp = 0.0, sq = 0.0;
        for (int32_t g = tid; g < ngroups; g += kThreads) {
            float lp[4], lq[4];
            load4<VEC>(prow, a.dt, g * 4, V, lp);
#pragma unroll
            for (int e = 0; e < 4; ++e) sp += (double)__builtin_amdgcn_exp2f(fmaf(lp[e], a.c2, -mp));
            if (has_children) {
                load4<VEC>(qrow, a.dt, g * 4, V, lq);
#pragma unroll
                for (int e = 0; e < 4; ++e) sq += (double)__builtin_amdgcn_exp2f(fmaf(lq[e], a.c2, -mq));
            }
        }
        sp = block_sum(sp, red);
        sq = has_children ? block_sum(sq, red) : 1.0;
        if (tid == 0) {
            st.lse2_p = (double)mp + log2(sp);
            st.lse2_q = (double)mq + log2(sq);
            st.S[0] = 1.0;
            st.nrej = 0;
            st.dead = sp > 0.0 ? 0 : 1;  // a row of -inf: nothing to accept, the draw gives token 0
            decision = -1;
        }
        __syncthreads();
        const float lp2 = (float)st.lse2_p, lq2 = (float)st.lse2_q;

        // the children in the order of their ranks
        for (int r = 0; r < kMaxRank; ++r) {
            const int32_t child = child_of_rank[r];
            if (child < 0) continue;                       // workgroup-uniform
            const int32_t x = a.draft_tokens[(int64_t)b * N + child];
            if (x < 0 || x >= V) continue;                 // a missing arrival is passed over
            if (tid == 0) {
                const int32_t j = st.nrej;
                const double p0 = exp2((double)widen(prow, a.dt, x) * a.c2d - st.lse2_p);
                const double q0 = exp2((double)widen(qrow, a.dt, x) * a.c2d - st.lse2_q);
                const double Pj = st.dead ? 0.0 : residual_weight(st, x, p0, q0, j);
                const double Qj = q0 / st.S[j];            // x was not rejected before: arrivals are distinct tokens
                uint32_t w[4];
                philox4x32((uint32_t)r, (uint32_t)ctx, (uint32_t)b, 2u, a.key0, a.key1, w);
                const double U = ((double)w[0] + 0.5) * 0x1p-32;
                if (Pj / Qj > U) {
                    decision = child;
                } else {
                    st.removed[j] = x;
                    st.S[j + 1] = st.S[j] - q0;
                }
            }
            __syncthreads();
            if (decision >= 0) break;
            // rejected: the normaliser of the next residual, one pass over both rows
            const int32_t j = st.nrej;
            double z = 0.0;
            if (!st.dead) {
                for (int32_t g = tid; g < ngroups; g += kThreads) {
                    float lp[4], lq[4];
                    load4<VEC>(prow, a.dt, g * 4, V, lp);
                    load4<VEC>(qrow, a.dt, g * 4, V, lq);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int32_t t = g * 4 + e;
                        if (t >= V) continue;
                        const double p0 = (double)__builtin_amdgcn_exp2f(fmaf(lp[e], a.c2, -lp2));
                        const double q0 = (double)__builtin_amdgcn_exp2f(fmaf(lq[e], a.c2, -lq2));
                        const double Pj = residual_weight(st, t, p0, q0, j);
                        bool gone = false;
                        for (int32_t i = 0; i < j; ++i) gone = gone || st.removed[i] == t;
                        const double d = Pj - (gone ? 0.0 : q0 / st.S[j]);
                        if (d > 0.0) z += d;
                    }
                }
            }
            z = block_sum(z, red);
            if (tid == 0) {
                st.Z[j + 1] = z;
                if (!(z > 0.0)) st.dead = 1;
                st.nrej = j + 1;
            }
            __syncthreads();
        }
        if (decision >= 0) {  // accepted: go on at the child's context
            const int32_t took = decision;
            if (tid == 0) out[len] = a.draft_tokens[(int64_t)b * N + took];
            ++len;
            node = took;
            ctx = took + 1;
            __syncthreads();  // `decision` is reset at the next context
            continue;
        }

        // the draw from what is left of P: race over the weights P_j(t), counter (i >> 2, ctx, b, 1)
        const int32_t level = st.nrej;
        const bool with_q = level > 0;
        if (tid == 0) count = 0;
        __syncthreads();
        double bs = -INFINITY;
        int32_t bi = -1;
        if (!st.dead) {
            float my_tau = kNone;
            for (int pass = 0; pass < 2; ++pass) {  // 0: a lower bound of the best score; 1: who can reach it
                if (pass == 1) my_tau = block_max(my_tau, red);
                for (int32_t g = tid; g < ngroups; g += kThreads) {
                    float lp[4], lq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    uint32_t w[4];
                    load4<VEC>(prow, a.dt, g * 4, V, lp);
                    if (with_q) load4<VEC>(qrow, a.dt, g * 4, V, lq);
                    philox4x32((uint32_t)g, (uint32_t)ctx, (uint32_t)b, 1u, a.key0, a.key1, w);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int32_t t = g * 4 + e;
                        if (t >= V) continue;
                        const double p0 = (double)__builtin_amdgcn_exp2f(fmaf(lp[e], a.c2, -lp2));
                        const double q0 = with_q ? (double)__builtin_amdgcn_exp2f(fmaf(lq[e], a.c2, -lq2)) : 0.0;
                        const float wt = (float)residual_weight(st, t, p0, q0, level);
                        if (!(wt > 0.0f)) continue;
                        const float s2 = __builtin_amdgcn_logf(wt) - log2_exponential(w[e]);
                        if (pass == 0) {
                            my_tau = fmaxf(my_tau, s2 - kLogErr);
                        } else if (s2 + kLogErr >= my_tau) {
                            const int32_t pos = atomicAdd(&count, 1);
                            if (pos < kListCap) { cand[pos] = t; cword[pos] = w[e]; }
                        }
                    }
                }
            }
            __syncthreads();
            const int32_t n = count;
            // the listed tokens (or, if the list overflowed, every token) with the exact exponential
            auto exact = [&](int32_t t, uint32_t word) {
                const double p0 = exp2((double)widen(prow, a.dt, t) * a.c2d - st.lse2_p);
                const double q0 = with_q ? exp2((double)widen(qrow, a.dt, t) * a.c2d - st.lse2_q) : 0.0;
                const double wt = residual_weight(st, t, p0, q0, level);
                const double v = ((double)word + 0.5) * 0x1p-32;
                return wt > 0.0 ? log(wt) - log(-log1p(-v)) : -INFINITY;
            };
            if (n <= kListCap) {
                for (int32_t k = tid; k < n; k += kThreads) {
                    const double s = exact(cand[k], cword[k]);
                    if (s > -INFINITY && (bi < 0 || s > bs || (s == bs && cand[k] < bi))) { bs = s; bi = cand[k]; }
                }
            } else {
                for (int32_t g = tid; g < ngroups; g += kThreads) {
                    uint32_t w[4];
                    philox4x32((uint32_t)g, (uint32_t)ctx, (uint32_t)b, 1u, a.key0, a.key1, w);
                    for (int e = 0; e < 4 && g * 4 + e < V; ++e) {
                        const double s = exact(g * 4 + e, w[e]);
                        if (s > -INFINITY && (bi < 0 || s > bs || (s == bs && g * 4 + e < bi))) { bs = s; bi = g * 4 + e; }
                    }
                }
            }
        }
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
            const double os = __shfl_xor(bs, off, kWave);
            const int32_t oi = __shfl_xor(bi, off, kWave);
            if (oi >= 0 && (bi < 0 || os > bs || (os == bs && oi < bi))) { bs = os; bi = oi; }
        }
        if ((tid & (kWave - 1)) == 0) { best_s[tid / kWave] = bs; best_i[tid / kWave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kWaves; ++w)
                if (best_i[w] >= 0 && (bi < 0 || best_s[w] > bs || (best_s[w] == bs && best_i[w] < bi))) {
                    bs = best_s[w];
                    bi = best_i[w];
                }
            out[len] = bi >= 0 ? bi : 0;  // nothing left of P: token 0 by convention
            a.accept_len[b] = len;
            a.accept_node[b] = node;
        }
        return;
    }
}

template <bool VEC>
__global__ void __launch_bounds__(kThreads) gsd_tree_walk_kernel(TreeArgs a) {
    walk_prompt<VEC>(a, blockIdx.x);
}

}  // namespace

extern "C" {

int ersd_gsd_verify_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t N,
                         int32_t V, const int32_t* parent, const int32_t* rank, const void* plan, size_t plan_bytes,
                         const int32_t* draft_tokens, float temperature, uint64_t seed, int32_t* accept_len,
                         int32_t* accept_node, int32_t* emitted, void* stream) {
    if (!draft_logits || !target_logits || !parent || !rank || !plan || !draft_tokens || !accept_len || !accept_node ||
        !emitted)
        return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (!(temperature > 0.0f) || !std::isfinite(temperature)) return ERSD_ERR_INVALID_ARG;
    if (((uintptr_t)draft_logits & 15) || ((uintptr_t)target_logits & 15) || ((uintptr_t)plan & 15))
        return ERSD_ERR_MISALIGNED;
    if (B < 1 || N < 1 || N > ERSD_MAX_ARRIVAL_TREE_NODES || V < 1 || V > (1 << 30)) return ERSD_ERR_INVALID_ARG;
    if ((int64_t)B * (N + 1) > 0x7fffffff) return ERSD_ERR_INVALID_ARG;
    const ersd_plan::PlanLayout pl = ersd_plan::plan_layout(N);
    if (plan_bytes < pl.total) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    TreeArgs a{};
    a.draft = static_cast<const char*>(draft_logits);
    a.target = static_cast<const char*>(target_logits);
    a.parent = parent;
    a.rank = rank;
    a.valid = reinterpret_cast<const int32_t*>(static_cast<const char*>(plan) + pl.valid);
    a.draft_tokens = draft_tokens;
    a.accept_len = accept_len;
    a.accept_node = accept_node;
    a.emitted = emitted;
    a.B = B;
    a.N = N;
    a.V = V;
    a.dt = (int)dt;
    a.c2d = 1.4426950408889634 / (double)temperature;
    a.c2 = (float)a.c2d;
    a.key0 = (uint32_t)(seed & 0xffffffffu);
    a.key1 = (uint32_t)(seed >> 32);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if ((V % 8) == 0) hipLaunchKernelGGL(gsd_tree_walk_kernel<true>, dim3((uint32_t)B), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(gsd_tree_walk_kernel<false>, dim3((uint32_t)B), dim3(kThreads), 0, s, a);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

}  // extern "C"
