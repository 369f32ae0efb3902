// libersd: verification by the comparison method, GSD (Section 2 of the paper; Algorithm 1 applied position by
// position as the text on the sequence strategy describes), for gfx950.  It exists to put a number on the paper's
// remark that verification by exponential races is simpler: on the same logits GSD needs the two softmax
// normalisers of every drafted position (one pass over all rows, an exponential per logit) and then a second,
// dependent pass over the rejected position's two rows to draw from the residual max(P - Q, 0).
//
//   normalisers : per (sequence, position) pair row and vocabulary split, every lane keeps a running maximum and a
//                 sum of 2^(z - max) in single precision (z = logit * log2(e) / T); lanes, wavefronts and splits
//                 are merged exactly in that form, the last step in double precision.
//   accept      : one thread per sequence walks the positions: P(x)/Q(x) > U with the uniform of the counter
//                 (0, j, b, 2); stores the first rejected position and its two normalisers.
//   residual    : the rows of that position again: weight max(p - q, 0) (or p after the last drafted position),
//                 score log2(weight) - log2(e) with e from the counter (i >> 2, a, b, 1).  Single-precision scores
//                 carry a margin for the cancellation in p - q; every token whose upper score reaches the best
//                 lower score is rescored in double precision, and the split's winner goes to the last kernel.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "ersd.h"
#include "ersd_philox.h"

namespace {

using ersd_philox::philox4x32;

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr int kListCap = 512;
constexpr float kNone = -3.0e38f;  // "no value yet": below every finite score, but finite so that differences are defined

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float widen(const char* row, int dt, int32_t i) {
    if (dt == ERSD_F32) return reinterpret_cast<const float*>(row)[i];
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(row)[i] << 16);
}

// running (maximum, sum of 2^(z - maximum)) of a stream of z; merging two of them is exact up to rounding
struct MaxSum {
    float m, s;
};
__device__ __forceinline__ void add_value(MaxSum& a, float z) {
    const float d = z - a.m;
    const float e = __builtin_amdgcn_exp2f(-fabsf(d));  // 2^-|d|; d = -inf (a masked logit) gives 0
    a.s = d > 0.0f ? fmaf(a.s, e, 1.0f) : a.s + e;
    a.m = fmaxf(a.m, z);
}
__device__ __forceinline__ MaxSum merge(const MaxSum& a, const MaxSum& b) {
    MaxSum o;
    o.m = fmaxf(a.m, b.m);
    o.s = a.s * __builtin_amdgcn_exp2f(a.m - o.m) + b.s * __builtin_amdgcn_exp2f(b.m - o.m);
    return o;
}
__device__ __forceinline__ MaxSum wave_merge(MaxSum v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        MaxSum o;
        o.m = __shfl_xor(v.m, off, kWave);
        o.s = __shfl_xor(v.s, off, kWave);
        v = merge(v, o);
    }
    return v;
}

__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Eight logits of one lane into the wavefront's running (maximum, per-lane sum): the maximum is kept uniform over
// the wavefront, so that it rises only a handful of times per row and the common case is one fused multiply-add,
// one 2^x and one addition per logit.
__device__ __forceinline__ void add_piece(float& m, float& s, const float (&l)[8], float c2) {
    float t[8], top = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        t[e] = fmaf(l[e], c2, -m);
        top = fmaxf(top, t[e]);
    }
    if (__builtin_amdgcn_ballot_w64(top > 0.0f) != 0) {  // rare: some lane saw a logit above the maximum
        float zm = m;  // the new maximum from the scaled logits themselves (top + m would cancel against the start value)
#pragma unroll
        for (int e = 0; e < 8; ++e) zm = fmaxf(zm, l[e] * c2);
        const float m_new = wave_max_f(zm);
        s *= __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = fmaf(l[e], c2, -m);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s += __builtin_amdgcn_exp2f(t[e]);
}

struct Geometry {
    int32_t B, k, V;
    int32_t S1;      // vocabulary splits of the normaliser pass
    int32_t chunk1;  // tokens per split (a multiple of 8)
    int32_t S3;      // splits of the residual pass
    int32_t chunk3;
};

struct NormArgs {
    const char* draft;
    const char* target;
    float4* partial;  // [row][split]: (max_q, sum_q, max_p, sum_p)
    Geometry g;
    float c2;         // log2(e) / T
};

template <int DT, bool VEC>
__global__ void __launch_bounds__(kThreads) gsd_normaliser_kernel(NormArgs a) {
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x / a.g.S1;  // (b, j), j < k
    const int32_t split = blockIdx.x % a.g.S1;
    const int64_t b = row / a.g.k;
    const int32_t j = (int32_t)(row % a.g.k);
    constexpr int es = DT == ERSD_F32 ? 4 : 2;
    const char* qrow = a.draft + (size_t)row * a.g.V * es;
    const char* prow = a.target + (size_t)(b * (a.g.k + 1) + j) * a.g.V * es;
    const int32_t begin = split * a.g.chunk1;
    const int32_t end = min(a.g.V, begin + a.g.chunk1);
    MaxSum q = {kNone, 0.0f}, p = {kNone, 0.0f};
    if (VEC) {
        constexpr int kTok = 16 / es;  // tokens per 128-bit piece
        constexpr int kUnroll = 4;     // pieces in flight per row and lane
        // the trip count is the same for every lane: the lanes of a wavefront meet inside add_piece
        for (int32_t tile = begin; tile < end; tile += kThreads * kTok * kUnroll) {
            const int32_t base = tile + tid * kTok;
            u32x4 rq[kUnroll], rp[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {  // unconditional loads from clamped addresses
                const int32_t i = base + u * kThreads * kTok;
                const int32_t c = i < end ? i : end - kTok;
                rq[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qrow + (size_t)c * es));
                rp[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(prow + (size_t)c * es));
            }
#pragma unroll
            for (int u = 0; u < kUnroll; u += (DT == ERSD_F32 ? 2 : 1)) {
                // a piece past the end re-read the last one: count it as masked (uniform control flow is kept
                // because the wavefront's maximum is found together)
                float lq[8], lp[8];
                if (DT == ERSD_F32) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const bool in = base + (u + h) * kThreads * kTok < end;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            lq[h * 4 + e] = in ? __uint_as_float(rq[u + h][e]) : -INFINITY;
                            lp[h * 4 + e] = in ? __uint_as_float(rp[u + h][e]) : -INFINITY;
                        }
                    }
                } else {
                    const bool in = base + u * kThreads * kTok < end;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        lq[2 * e] = in ? __uint_as_float(rq[u][e] << 16) : -INFINITY;
                        lq[2 * e + 1] = in ? __uint_as_float(rq[u][e] & 0xffff0000u) : -INFINITY;
                        lp[2 * e] = in ? __uint_as_float(rp[u][e] << 16) : -INFINITY;
                        lp[2 * e + 1] = in ? __uint_as_float(rp[u][e] & 0xffff0000u) : -INFINITY;
                    }
                }
                add_piece(q.m, q.s, lq, a.c2);
                add_piece(p.m, p.s, lp, a.c2);
            }
        }
        // the maximum is uniform over the wavefront: add the lanes' sums
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
            q.s += __shfl_xor(q.s, off, kWave);
            p.s += __shfl_xor(p.s, off, kWave);
        }
    } else {
        for (int32_t i = begin + tid; i < end; i += kThreads) {
            add_value(q, widen(qrow, DT, i) * a.c2);
            add_value(p, widen(prow, DT, i) * a.c2);
        }
    }
    if (!VEC) {
        q = wave_merge(q);
        p = wave_merge(p);
    }
    __shared__ MaxSum sq[kWaves], sp[kWaves];
    if ((tid & (kWave - 1)) == 0) { sq[tid / kWave] = q; sp[tid / kWave] = p; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w) { q = merge(q, sq[w]); p = merge(p, sp[w]); }
        a.partial[row * a.g.S1 + split] = make_float4(q.m, q.s, p.m, p.s);
    }
}

struct Verdict {  // what the accept kernel hands to the residual pass, per sequence
    double lse2_p, lse2_q;  // normalisers (log2 units) of the position the next token is drawn at
    int32_t a;              // that position = number of accepted tokens
    int32_t pad;
};

struct AcceptArgs {
    const char* draft;
    const char* target;
    const float4* partial;
    const int32_t* draft_tokens;
    int32_t* accept_len;
    Verdict* verdict;
    Geometry g;
    int dt;
    double c2;  // log2(e) / T in double precision
    uint32_t key0, key1;
};

// log2 of the sum over a row from its split partials.  The rescaling 2^(m_s - m) and the final logarithm use the
// single-precision hardware functions (a few 1e-7 of relative error, like the partial sums themselves); the sum
// is kept in double precision.
__device__ void row_normalisers(const float4* part, int32_t S, double& lse2_q, double& lse2_p) {
    float mq = -INFINITY, mp = -INFINITY;
    for (int32_t s = 0; s < S; ++s) {
        if (part[s].y > 0.0f) mq = fmaxf(mq, part[s].x);
        if (part[s].w > 0.0f) mp = fmaxf(mp, part[s].z);
    }
    double sq = 0.0, sp = 0.0;
    for (int32_t s = 0; s < S; ++s) {
        if (part[s].y > 0.0f) sq += (double)(part[s].y * __builtin_amdgcn_exp2f(part[s].x - mq));
        if (part[s].w > 0.0f) sp += (double)(part[s].w * __builtin_amdgcn_exp2f(part[s].z - mp));
    }
    lse2_q = sq > 0.0 ? (double)mq + (double)__builtin_amdgcn_logf((float)sq) : -INFINITY;
    lse2_p = sp > 0.0 ? (double)mp + (double)__builtin_amdgcn_logf((float)sp) : -INFINITY;
}

// One workgroup per sequence: the positions are tested in parallel, then the first rejection is found.
__global__ void __launch_bounds__(kThreads) gsd_accept_kernel(AcceptArgs a) {
    const int32_t b = blockIdx.x, tid = threadIdx.x;
    const int es = a.dt == ERSD_F32 ? 4 : 2;
    __shared__ int32_t first_reject;
    if (tid == 0) first_reject = a.g.k;
    __syncthreads();
    for (int32_t j = tid; j < a.g.k; j += kThreads) {
        const int64_t row = (int64_t)b * a.g.k + j;
        const int32_t x = a.draft_tokens[row];
        bool ok = x >= 0 && x < a.g.V;  // not a token: rejected without touching the rows
        if (ok) {
            double lq, lp;
            row_normalisers(a.partial + row * a.g.S1, a.g.S1, lq, lp);
            const char* qrow = a.draft + (size_t)row * a.g.V * es;
            const char* prow = a.target + (size_t)((int64_t)b * (a.g.k + 1) + j) * a.g.V * es;
            // P(x) / Q(x) > U
            const double ratio =
                exp2(((double)widen(prow, a.dt, x) * a.c2 - lp) - ((double)widen(qrow, a.dt, x) * a.c2 - lq));
            uint32_t w[4];
            philox4x32(0u, (uint32_t)j, (uint32_t)b, 2u, a.key0, a.key1, w);
            ok = ratio > ((double)w[0] + 0.5) * 0x1p-32;
        }
        if (!ok) atomicMin(&first_reject, j);
    }
    __syncthreads();
    if (tid == 0) {
        const int32_t acc = first_reject;
        a.accept_len[b] = acc;
        Verdict v;
        v.a = acc;
        v.pad = 0;
        v.lse2_p = v.lse2_q = 0.0;  // not used when every token was accepted: a draw from P needs no normaliser
        if (acc < a.g.k) row_normalisers(a.partial + ((int64_t)b * a.g.k + acc) * a.g.S1, a.g.S1, v.lse2_q, v.lse2_p);
        a.verdict[b] = v;
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

struct Winner {
    double score;  // natural-log units; -inf: no token with a positive weight
    int32_t idx;
    int32_t pad;
};

struct ResidualArgs {
    const char* draft;
    const char* target;
    const Verdict* verdict;
    Winner* winner;  // [b][split]
    Geometry g;
    int dt;
    float c2;
    double T;
    uint32_t key0, key1;
};

__device__ __forceinline__ bool better(double s, int32_t i, double bs, int32_t bi) {
    return bi < 0 || s > bs || (s == bs && i < bi);
}

// weight and score of token i exactly as the definition says, in double precision
__device__ double exact_score(const ResidualArgs& a, const char* qrow, const char* prow, double lse_p, double lse_q,
                              int32_t i, uint32_t word) {
    const double v = ((double)word + 0.5) * 0x1p-32;
    const double lne = log(-log1p(-v));
    if (!qrow) return (double)widen(prow, a.dt, i) / a.T - lne;  // a draw from P: ln p up to a constant
    const double p = exp((double)widen(prow, a.dt, i) / a.T - lse_p);
    const double q = exp((double)widen(qrow, a.dt, i) / a.T - lse_q);
    const double w = p - q > 0.0 ? p - q : 0.0;
    return log(w) - lne;
}

// Relative slack of the single-precision weights: rounding of the scaled logit (about 30 * 2^-24 in the exponent),
// of 2^x, and the error of the normalisers.  The lower and upper scores below use w -+ kDelta (p + q).
constexpr float kDelta = 1.0e-5f;
constexpr float kLogErr = 0x1p-5f + 0x1p-10f;  // log2_exponential (2^-7), v_log_f32, and the final subtraction

// four consecutive logits of a row (i a multiple of 4, in range): one 8- or 16-byte load when the row allows it
template <bool VEC>
__device__ __forceinline__ void load4(const char* row, int dt, int32_t i, int32_t end, float out[4]) {
    if (VEC) {
        if (dt == ERSD_F32) {
            const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + (size_t)i * 4));
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = __uint_as_float(r[e]);
        } else {
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            const u32x2 r = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(row + (size_t)i * 2));
            out[0] = __uint_as_float(r[0] << 16); out[1] = __uint_as_float(r[0] & 0xffff0000u);
            out[2] = __uint_as_float(r[1] << 16); out[3] = __uint_as_float(r[1] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = i + e < end ? widen(row, dt, i + e) : -INFINITY;
    }
}

// single-precision upper and lower score (log2 units) of one token; false if it cannot win
__device__ __forceinline__ bool fast_scores(bool residual, float lp, float lq, float c2, float lp2, float lq2, uint32_t word,
                                            float& up, float& down) {
    down = -INFINITY;
    if (residual) {
        const float p = __builtin_amdgcn_exp2f(fmaf(lp, c2, -lp2));
        const float q = __builtin_amdgcn_exp2f(fmaf(lq, c2, -lq2));
        const float slack = kDelta * (p + q);
        const float hi = p - q + slack, lo = p - q - slack;
        if (!(hi > 0.0f)) return false;
        const float l2e = log2_exponential(word);
        up = __builtin_amdgcn_logf(hi) - l2e + kLogErr;
        if (lo > 0.0f) down = __builtin_amdgcn_logf(lo) - l2e - kLogErr;
    } else {  // a draw from P: the score is the scaled logit minus log2 e, no normaliser
        const float z = lp * c2;
        if (!(z > -INFINITY)) return false;
        const float l2e = log2_exponential(word);
        const float margin = kLogErr + fabsf(z) * 0x1p-20f;
        up = z - l2e + margin;
        down = z - l2e - margin;
    }
    return true;
}

template <bool VEC>
__global__ void __launch_bounds__(kThreads) gsd_residual_kernel(ResidualArgs a) {
    const int tid = threadIdx.x;
    const int32_t b = blockIdx.x / a.g.S3, split = blockIdx.x % a.g.S3;
    const Verdict v = a.verdict[b];
    const int es = a.dt == ERSD_F32 ? 4 : 2;
    const bool residual = v.a < a.g.k;
    const char* prow = a.target + (size_t)((int64_t)b * (a.g.k + 1) + v.a) * a.g.V * es;
    const char* qrow = residual ? a.draft + (size_t)((int64_t)b * a.g.k + v.a) * a.g.V * es : nullptr;
    const int32_t begin = split * a.g.chunk3, end = min(a.g.V, begin + a.g.chunk3);
    const float lp2 = (float)v.lse2_p, lq2 = (float)v.lse2_q;

    __shared__ float tau;
    __shared__ int32_t count;
    __shared__ int32_t cand[kListCap];
    __shared__ uint32_t cword[kListCap];
    __shared__ double red_s[kWaves];
    __shared__ int32_t red_i[kWaves];
    __shared__ float red_t[kWaves];
    if (tid == 0) count = 0;

    // start from a lower bound of the best score: the best lower score among every lane's first group
    float my_tau = kNone;
    {
        const int32_t g = (begin >> 2) + tid;
        if (g * 4 < end) {
            uint32_t w[4];
            float lp[4], lq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            philox4x32((uint32_t)g, (uint32_t)v.a, (uint32_t)b, 1u, a.key0, a.key1, w);
            load4<VEC>(prow, a.dt, g * 4, end, lp);
            if (residual) load4<VEC>(qrow, a.dt, g * 4, end, lq);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float up, down;
                if (g * 4 + e < end && fast_scores(residual, lp[e], lq[e], a.c2, lp2, lq2, w[e], up, down))
                    my_tau = fmaxf(my_tau, down);
            }
        }
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) my_tau = fmaxf(my_tau, __shfl_xor(my_tau, off, kWave));
        if ((tid & (kWave - 1)) == 0) red_t[tid / kWave] = my_tau;
        __syncthreads();
        for (int w = 0; w < kWaves; ++w) my_tau = fmaxf(my_tau, red_t[w]);
        if (tid == 0) tau = my_tau;
        __syncthreads();
    }

    // every lane takes groups of four consecutive tokens (one generator call)
    for (int32_t g = (begin >> 2) + tid; g * 4 < end; g += kThreads) {
        uint32_t w[4];
        float lp[4], lq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        load4<VEC>(prow, a.dt, g * 4, end, lp);
        if (residual) load4<VEC>(qrow, a.dt, g * 4, end, lq);
        philox4x32((uint32_t)g, (uint32_t)v.a, (uint32_t)b, 1u, a.key0, a.key1, w);
        my_tau = fmaxf(my_tau, __hip_atomic_load(&tau, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t i = g * 4 + e;
            float up, down;
            if (i >= end || !fast_scores(residual, lp[e], lq[e], a.c2, lp2, lq2, w[e], up, down)) continue;
            if (up >= my_tau) {
                const int32_t pos = atomicAdd(&count, 1);
                if (pos < kListCap) { cand[pos] = i; cword[pos] = w[e]; }
                if (down > my_tau) {
                    my_tau = down;
                    __hip_atomic_fetch_max(&tau, down, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
        }
    }
    __syncthreads();
    const double lse_p = v.lse2_p * 0.6931471805599453, lse_q = v.lse2_q * 0.6931471805599453;
    double bs = -INFINITY;
    int32_t bi = -1;
    const int32_t n = count;
    if (n <= kListCap) {  // the listed tokens, exactly
        for (int32_t t = tid; t < n; t += kThreads) {
            const double s = exact_score(a, qrow, prow, lse_p, lse_q, cand[t], cword[t]);
            if (s > -INFINITY && better(s, cand[t], bs, bi)) { bs = s; bi = cand[t]; }
        }
    } else {  // rare: the list overflowed; every token of the split, exactly
        for (int32_t g = (begin >> 2) + tid; g * 4 < end; g += kThreads) {
            uint32_t w[4];
            philox4x32((uint32_t)g, (uint32_t)v.a, (uint32_t)b, 1u, a.key0, a.key1, w);
            for (int e = 0; e < 4; ++e) {
                const int32_t i = g * 4 + e;
                if (i >= end) break;
                const double s = exact_score(a, qrow, prow, lse_p, lse_q, i, w[e]);
                if (s > -INFINITY && better(s, i, bs, bi)) { bs = s; bi = i; }
            }
        }
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const double os = __shfl_xor(bs, off, kWave);
        const int32_t oi = __shfl_xor(bi, off, kWave);
        if (oi >= 0 && better(os, oi, bs, bi)) { bs = os; bi = oi; }
    }
    if ((tid & (kWave - 1)) == 0) { red_s[tid / kWave] = bs; red_i[tid / kWave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kWaves; ++w)
            if (red_i[w] >= 0 && better(red_s[w], red_i[w], bs, bi)) { bs = red_s[w]; bi = red_i[w]; }
        Winner o;
        o.score = bi >= 0 ? bs : -INFINITY;
        o.idx = bi;
        o.pad = 0;
        a.winner[(int64_t)b * a.g.S3 + split] = o;
    }
}

__global__ void __launch_bounds__(kThreads) gsd_pick_kernel(const Winner* winner, int32_t B, int32_t S3,
                                                            int32_t* next_token) {
    const int32_t b = blockIdx.x * kThreads + threadIdx.x;
    if (b >= B) return;
    double bs = -INFINITY;
    int32_t bi = -1;
    for (int32_t s = 0; s < S3; ++s) {
        const Winner w = winner[(int64_t)b * S3 + s];
        if (w.idx >= 0 && better(w.score, w.idx, bs, bi)) { bs = w.score; bi = w.idx; }
    }
    next_token[b] = bi >= 0 ? bi : 0;  // no token with a positive weight: token 0 by convention
}

// ---------------------------------------------------------------------------------------------- host side
int32_t ceil_div(int64_t a, int64_t b) { return (int32_t)((a + b - 1) / b); }

bool make_geometry(int32_t B, int32_t k, int32_t V, Geometry& g) {
    if (B < 1 || k < 1 || V < 1 || V > 0x7fff0000 || k == 0x7fffffff) return false;
    if ((int64_t)B * (k + 1) > 0x7fffffff / 64) return false;  // grids: rows times splits stay in int32
    g.B = B;
    g.k = k;
    g.V = V;
    const int64_t rows = (int64_t)B * k;
    // enough workgroups to fill the chip several times over, each with at least 8192 tokens per row
    int32_t s1 = ceil_div(4096, rows);
    const int32_t most1 = ceil_div(V, 8192);
    if (s1 > most1) s1 = most1;
    if (s1 > 64) s1 = 64;
    if (s1 < 1) s1 = 1;
    g.chunk1 = ceil_div(ceil_div(V, s1), 8) * 8;
    g.S1 = ceil_div(V, g.chunk1);
    int32_t s3 = ceil_div(1024, B);
    const int32_t most3 = ceil_div(V, 4096);
    if (s3 > most3) s3 = most3;
    if (s3 > 64) s3 = 64;
    if (s3 < 1) s3 = 1;
    g.chunk3 = ceil_div(ceil_div(V, s3), 8) * 8;
    g.S3 = ceil_div(V, g.chunk3);
    return true;
}

size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

struct Layout {
    size_t partial, verdict, winner, total;
};
Layout make_layout(const Geometry& g) {
    Layout l;
    l.partial = 0;
    l.verdict = align16(l.partial + (size_t)g.B * g.k * g.S1 * sizeof(float4));
    l.winner = align16(l.verdict + (size_t)g.B * sizeof(Verdict));
    l.total = align16(l.winner + (size_t)g.B * g.S3 * sizeof(Winner));
    return l;
}

}  // namespace

extern "C" {

size_t ersd_gsd_workspace_bytes(int32_t B, int32_t k, int32_t V, ersd_dtype dt) {
    Geometry g;
    if ((dt != ERSD_F32 && dt != ERSD_BF16) || !make_geometry(B, k, V, g)) return 0;
    return make_layout(g).total;
}

int ersd_gsd_verify(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t k, int32_t V,
                    const int32_t* draft_tokens, float temperature, uint64_t seed, int32_t* accept_len,
                    int32_t* next_token, void* workspace, size_t workspace_bytes, void* stream) {
    if (!draft_logits || !target_logits || !draft_tokens || !accept_len || !next_token || !workspace)
        return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (!(temperature > 0.0f) || !std::isfinite(temperature)) return ERSD_ERR_INVALID_ARG;
    if (((uintptr_t)draft_logits & 15) || ((uintptr_t)target_logits & 15) || ((uintptr_t)workspace & 15))
        return ERSD_ERR_MISALIGNED;
    Geometry g;
    if (!make_geometry(B, k, V, g)) return ERSD_ERR_INVALID_ARG;
    const Layout l = make_layout(g);
    if (workspace_bytes < l.total) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    char* base = static_cast<char*>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const double c2 = 1.4426950408889634 / (double)temperature;

    NormArgs na;
    na.draft = static_cast<const char*>(draft_logits);
    na.target = static_cast<const char*>(target_logits);
    na.partial = reinterpret_cast<float4*>(base + l.partial);
    na.g = g;
    na.c2 = (float)c2;
    const dim3 grid1((uint32_t)((int64_t)B * k * g.S1)), block(kThreads);
    const bool vec = (V % 8) == 0;
    if (dt == ERSD_F32) {
        if (vec) hipLaunchKernelGGL((gsd_normaliser_kernel<ERSD_F32, true>), grid1, block, 0, s, na);
        else hipLaunchKernelGGL((gsd_normaliser_kernel<ERSD_F32, false>), grid1, block, 0, s, na);
    } else {
        if (vec) hipLaunchKernelGGL((gsd_normaliser_kernel<ERSD_BF16, true>), grid1, block, 0, s, na);
        else hipLaunchKernelGGL((gsd_normaliser_kernel<ERSD_BF16, false>), grid1, block, 0, s, na);
    }

    AcceptArgs aa;
    aa.draft = na.draft;
    aa.target = na.target;
    aa.partial = na.partial;
    aa.draft_tokens = draft_tokens;
    aa.accept_len = accept_len;
    aa.verdict = reinterpret_cast<Verdict*>(base + l.verdict);
    aa.g = g;
    aa.dt = (int)dt;
    aa.c2 = c2;
    aa.key0 = (uint32_t)(seed & 0xffffffffu);
    aa.key1 = (uint32_t)(seed >> 32);
    hipLaunchKernelGGL(gsd_accept_kernel, dim3((uint32_t)B), block, 0, s, aa);

    ResidualArgs ra;
    ra.draft = na.draft;
    ra.target = na.target;
    ra.verdict = aa.verdict;
    ra.winner = reinterpret_cast<Winner*>(base + l.winner);
    ra.g = g;
    ra.dt = (int)dt;
    ra.c2 = (float)c2;
    ra.T = (double)temperature;
    ra.key0 = aa.key0;
    ra.key1 = aa.key1;
    if (vec) hipLaunchKernelGGL(gsd_residual_kernel<true>, dim3((uint32_t)((int64_t)B * g.S3)), block, 0, s, ra);
    else hipLaunchKernelGGL(gsd_residual_kernel<false>, dim3((uint32_t)((int64_t)B * g.S3)), block, 0, s, ra);
    hipLaunchKernelGGL(gsd_pick_kernel, dim3((uint32_t)((B + kThreads - 1) / kThreads)), block, 0, s, ra.winner, B, g.S3,
                       next_token);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

}  // extern "C"
