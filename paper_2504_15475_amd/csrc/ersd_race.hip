// libersd: exponential-race verification kernels for gfx950 (MI355X) and their C ABI.
//
// One race = one pass over a draft row and a target row that share their exponentials (Section 3 of the
// paper: the same realisation of e decides argmin e_i/Q(i) and argmin e_i/P(i)).  The winner is defined
// on fp64 scores  logit/T - ln e_i  (lowest index on exact ties).  Evaluating that for every token would
// be bound by fp64 transcendental code, so the streaming kernel is a FILTER followed by an exact stage:
//
//   stream  : per token, Philox word x -> a cheap fp32 UPPER bound of the score (log2 units):
//               -log2 e <= -log2 v = 32 - log2(x + 1/2) <= 159 - bits(float(x)) * 2^-23
//             (e = -ln(1-v) >= v, and log2(1+f) >= f on [0,1] makes the float bit pattern a lower bound of
//             log2).  A token is looked at again only if its bound reaches tau, a running LOWER bound
//             of the row maximum.
//   refine  : for those few tokens an fp32 score with a proven error margin, using v_log_f32; tokens
//             that can still be the maximum are appended to a candidate list in LDS and raise tau.
//   exact   : after the stream, the candidates (a few dozen per row) are scored in fp64 exactly as the
//             definition says and reduced with the (score, lowest index) order.
//
// Since tau never exceeds the true row maximum and the bounds are one-sided, the true winner (and every
// token tied with it) is always among the candidates, so the result is the fp64 argmax.
//
// Vocabulary splits: a row may be cut into `nsplit` chunks handled by different workgroups; each writes
// one (score, index) partial per side, combined in index order by the finishing kernel, which also
// computes the accept lengths (first-mismatch scan, best draft, tree ancestor walk).

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>

#include "ersd.h"

namespace {

constexpr int kThreads = 256;                       // 4 wavefronts per workgroup
constexpr int kTokPerThread = 8;                    // two Philox calls, 16 B of bf16 / 32 B of fp32 per side
constexpr int kTokPerIter = kThreads * kTokPerThread;
constexpr int kListCap = 1024;                      // candidate slots per side per workgroup
constexpr int kMaxSplit = 64;
constexpr int kWave = 64;

constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

struct Partial {
    double score;
    int32_t idx;
    int32_t pad;
};

struct RaceArgs {
    const char* draft;
    const char* target;
    Partial* partials;  // [row][side][split]
    int32_t V;
    int32_t kd;      // draft rows per sequence (k, or N for a tree)
    int32_t kt;      // target rows per sequence (k + 1, or N)
    int32_t m;       // drafts per prompt
    int32_t nsplit;
    int32_t chunk;   // tokens per split, a multiple of kTokPerIter
    uint32_t key0, key1;
    float c2;        // log2(e) / T
    double T;
};

// ------------------------------------------------------------------------------------------ Philox4x32-10
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ------------------------------------------------------------------------------------------ exact score
// The definition, in double precision: v = (x + 1/2) 2^-32, e = -log1p(-v), score = logit/T - ln e.
__device__ __noinline__ double exact_score(float logit, double T, uint32_t x) {
    const double v = ((double)x + 0.5) * 0x1p-32;
    const double e = -log1p(-v);
    return (double)logit / T - log(e);
}

__device__ __forceinline__ float widen_elem(const char* row, int dt, int32_t i) {
    if (dt == ERSD_F32) return reinterpret_cast<const float*>(row)[i];
    const uint32_t bits = (uint32_t)reinterpret_cast<const uint16_t*>(row)[i] << 16;
    return __uint_as_float(bits);
}

__device__ __forceinline__ double exact_score_at(const char* row, int dt, int32_t i, const RaceArgs& a,
                                                 uint32_t c1, uint32_t c2, uint32_t c3) {
    uint32_t w[4];
    philox4x32_10((uint32_t)i >> 2, c1, c2, c3, a.key0, a.key1, w);
    return exact_score(widen_elem(row, dt, i), a.T, w[i & 3]);
}

// (score, index) order: larger score first, then lower index.
__device__ __forceinline__ bool better(double s, int32_t i, double bs, int32_t bi) {
    return s > bs || (s == bs && i < bi);
}

// Workgroup argmax; every thread passes its own best (idx < 0 = none).  Result valid in thread 0.
__device__ void block_argmax(double& s, int32_t& i, double* lds_s, int32_t* lds_i) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const double os = __shfl_xor(s, off, kWave);
        const int32_t oi = __shfl_xor(i, off, kWave);
        if (oi >= 0 && (i < 0 || better(os, oi, s, i))) { s = os; i = oi; }
    }
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) { lds_s[wave] = s; lds_i[wave] = i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / kWave; ++w)
            if (lds_i[w] >= 0 && (i < 0 || better(lds_s[w], lds_i[w], s, i))) { s = lds_s[w]; i = lds_i[w]; }
    }
    __syncthreads();
}

// Row geometry shared by both race kernels.
struct RowCtx {
    const char* qrow;  // draft row or nullptr (bonus position)
    const char* prow;  // target row
    uint32_t c1, c2, c3;
    int32_t begin, end;  // token range of this split
    int64_t row;
    int32_t split;
};

template <int DT>
__device__ __forceinline__ RowCtx make_ctx(const RaceArgs& a) {
    RowCtx c;
    const int64_t blk = blockIdx.x;
    c.split = (int32_t)(blk % a.nsplit);
    c.row = blk / a.nsplit;                  // target row index = seq * kt + j
    const int64_t seq = c.row / a.kt;        // b * m + d
    const int32_t j = (int32_t)(c.row % a.kt);
    const size_t es = DT == ERSD_F32 ? 4 : 2;
    c.prow = a.target + (size_t)c.row * (size_t)a.V * es;
    c.qrow = j < a.kd ? a.draft + (size_t)(seq * a.kd + j) * (size_t)a.V * es : nullptr;
    c.c1 = (uint32_t)j;
    c.c2 = (uint32_t)(seq / a.m);
    c.c3 = (uint32_t)(seq % a.m);
    c.begin = c.split * a.chunk;
    const int64_t e = (int64_t)c.begin + a.chunk;
    c.end = e < a.V ? (int32_t)e : a.V;
    return c;
}

__device__ __forceinline__ void store_partial(const RaceArgs& a, const RowCtx& c, int side, double s, int32_t i) {
    Partial p;
    p.score = s;
    p.idx = i;
    p.pad = 0;
    a.partials[((size_t)c.row * 2 + side) * a.nsplit + c.split] = p;
}

// Exact scan of one side of a split: every token scored in fp64.  Used by the reference kernel and as the
// fallback when a candidate list overflows.
template <int DT>
__device__ void exhaustive_side(const RaceArgs& a, const RowCtx& c, const char* row, int side,
                                double* lds_s, int32_t* lds_i) {
    double bs = -INFINITY;
    int32_t bi = -1;
    const int32_t g0 = c.begin >> 2, g1 = (c.end + 3) >> 2;  // c.begin is a multiple of 4
    for (int32_t g = g0 + (int32_t)threadIdx.x; g < g1; g += kThreads) {
        uint32_t w[4];
        philox4x32_10((uint32_t)g, c.c1, c.c2, c.c3, a.key0, a.key1, w);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t i = g * 4 + e;
            if (i < c.end) {
                const double s = exact_score(widen_elem(row, DT, i), a.T, w[e]);
                if (bi < 0 || s > bs) { bs = s; bi = i; }  // increasing i per thread: ties keep the lower index
            }
        }
    }
    block_argmax(bs, bi, lds_s, lds_i);
    if (threadIdx.x == 0) store_partial(a, c, side, bs, bi);
}

template <int DT>
__global__ void __launch_bounds__(kThreads) race_exhaustive_kernel(RaceArgs a) {
    __shared__ double lds_s[kThreads / kWave];
    __shared__ int32_t lds_i[kThreads / kWave];
    const RowCtx c = make_ctx<DT>(a);
    if (c.qrow) exhaustive_side<DT>(a, c, c.qrow, 0, lds_s, lds_i);
    exhaustive_side<DT>(a, c, c.prow, 1, lds_s, lds_i);
}

// ------------------------------------------------------------------------------------------ filtered kernel
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct Raw {  // 8 logits as loaded: bf16 -> a only (4 dwords); fp32 (or element loads) -> a, b
    u32x4 a, b;
};

constexpr uint32_t kNegInfF32 = 0xFF800000u, kNegInfBf16x2 = 0xFF80FF80u;

// RAWF32: registers hold fp32 bit patterns (fp32 rows, or rows read element by element).
template <int DT, bool VEC>
__device__ __forceinline__ Raw load_raw(const char* row, int32_t i0, int32_t end) {
    Raw r;
    if (VEC) {
        if (i0 >= end) {
            const uint32_t f = DT == ERSD_BF16 ? kNegInfBf16x2 : kNegInfF32;
            r.a = u32x4{f, f, f, f};
            r.b = r.a;
        } else if (DT == ERSD_BF16) {
            r.a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + (size_t)i0 * 2));
            r.b = r.a;
        } else {
            const u32x4* p = reinterpret_cast<const u32x4*>(row + (size_t)i0 * 4);
            r.a = __builtin_nontemporal_load(p);
            r.b = __builtin_nontemporal_load(p + 1);
        }
    } else {
        uint32_t f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int32_t i = i0 + e;
            f[e] = i < end ? __float_as_uint(widen_elem(row, DT, i)) : kNegInfF32;
        }
        r.a = u32x4{f[0], f[1], f[2], f[3]};
        r.b = u32x4{f[4], f[5], f[6], f[7]};
    }
    return r;
}

template <bool RAWF32>
__device__ __forceinline__ void unpack(const Raw& r, float l[8]) {
    if (RAWF32) {
        l[0] = __uint_as_float(r.a.x); l[1] = __uint_as_float(r.a.y);
        l[2] = __uint_as_float(r.a.z); l[3] = __uint_as_float(r.a.w);
        l[4] = __uint_as_float(r.b.x); l[5] = __uint_as_float(r.b.y);
        l[6] = __uint_as_float(r.b.z); l[7] = __uint_as_float(r.b.w);
    } else {
        const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            l[2 * e] = __uint_as_float(w[e] << 16);
            l[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
    }
}

// Upper bound of -log2 e from the word x alone (see file header); slack below is added to tau instead.
__device__ __forceinline__ float gumbel2_upper(uint32_t x) {
    const float xf = (float)x;
    return fmaf((float)(int32_t)__float_as_uint(xf), -0x1p-23f, 159.0f);
}

// log2 of e = -ln(1 - v) in fp32.  |error| < 2^-7 given v_log_f32 within a few ulp (checked on device by
// the test suite); callers use kRefineErr = 2^-5.
__device__ __forceinline__ float log2_exponential(uint32_t x) {
    if (x < (1u << 23)) {  // v < 2^-9, exact in fp32: series of -ln(1-v)
        const float v = ((float)x + 0.5f) * 0x1p-32f;
        const float poly = fmaf(v, fmaf(v, fmaf(v, fmaf(v, 0.2f, 0.25f), 0.33333334f), 0.5f), 1.0f);
        return __builtin_amdgcn_logf(v * poly);
    }
    // 1 - v = (~x + 1/2) 2^-32 <= 1 - 2^-9, so -log2(1-v) >= 2.8e-3 and the subtraction keeps ~9 bits
    const float y = (float)(~x) + 0.5f;
    const float e2 = 32.0f - __builtin_amdgcn_logf(y);
    return __builtin_amdgcn_logf(e2) - 0.5287663729f;  // + log2(ln 2)
}

constexpr float kRefineErr = 0x1p-5f;
constexpr float kRelErr = 0x1p-20f;
constexpr float kUpperSlack = 0x1p-10f;

__device__ __forceinline__ int32_t ordered_int(float f) {
    const int32_t i = __float_as_int(f);
    return i >= 0 ? i : i ^ 0x7fffffff;
}
__device__ __forceinline__ float from_ordered_int(int32_t i) {
    return __int_as_float(i >= 0 ? i : i ^ 0x7fffffff);
}
__device__ __forceinline__ float with_margin(float tau) { return tau - fmaf(fabsf(tau), kRelErr, kUpperSlack); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

struct Lds {
    int32_t tau[2];      // ordered-int encoding of the workgroup's lower bound, per side
    int32_t count[2];    // candidates appended (may exceed kListCap: overflow)
    int32_t list[2][kListCap];
    double red_s[kThreads / kWave];
    int32_t red_i[kThreads / kWave];
};

// One side's refine step for one token of one lane.
__device__ __forceinline__ void refine_token(float logit, float l2e, float c2, int32_t idx, float& tau, Lds& lds,
                                             int side) {
    const float s2 = fmaf(logit, c2, -l2e);
    const float err = fmaf(fabsf(s2), kRelErr, kRefineErr);
    if (s2 > -INFINITY && s2 + err >= tau) {
        const int32_t pos = atomicAdd(&lds.count[side], 1);
        if (pos < kListCap) lds.list[side][pos] = idx;
        tau = fmaxf(tau, s2 - err);
    }
}

template <int DT, bool VEC, bool HASQ>
__device__ void race_filtered_body(const RaceArgs& a, const RowCtx& c, Lds& lds) {
    constexpr bool RAWF32 = (DT == ERSD_F32) || !VEC;
    const int tid = threadIdx.x;
    const float c2 = a.c2;

    if (tid < 2) {
        lds.tau[tid] = ordered_int(-3.0e38f);
        lds.count[tid] = 0;
    }
    __syncthreads();

    // Bootstrap: a lower bound of the maximum from the first two tokens of every lane's first group.
    float tauq = -3.0e38f, taup = -3.0e38f;
    {
        const int32_t i0 = c.begin + tid * kTokPerThread;
        if (i0 < c.end) {
            uint32_t w[4];
            philox4x32_10((uint32_t)i0 >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, w);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                if (i0 + e < c.end) {
                    const float l2e = log2_exponential(w[e]);
                    const float sp = fmaf(widen_elem(c.prow, DT, i0 + e), c2, -l2e);
                    if (sp > -INFINITY) taup = fmaxf(taup, sp - fmaf(fabsf(sp), kRelErr, kRefineErr));
                    if (HASQ) {
                        const float sq = fmaf(widen_elem(c.qrow, DT, i0 + e), c2, -l2e);
                        if (sq > -INFINITY) tauq = fmaxf(tauq, sq - fmaf(fabsf(sq), kRelErr, kRefineErr));
                    }
                }
            }
        }
        taup = wave_max(taup);
        if (HASQ) tauq = wave_max(tauq);
        if ((tid & (kWave - 1)) == 0) {
            atomicMax(&lds.tau[1], ordered_int(taup));
            if (HASQ) atomicMax(&lds.tau[0], ordered_int(tauq));
        }
        __syncthreads();
        taup = from_ordered_int(lds.tau[1]);
        if (HASQ) tauq = from_ordered_int(lds.tau[0]);
    }

    Raw rq, rp;
    {
        const int32_t i0 = c.begin + tid * kTokPerThread;
        rp = load_raw<DT, VEC>(c.prow, i0, c.end);
        if (HASQ) rq = load_raw<DT, VEC>(c.qrow, i0, c.end);
    }
    for (int32_t base = c.begin; base < c.end; base += kTokPerIter) {
        const int32_t i0 = base + tid * kTokPerThread;
        Raw nq, np;
        {
            const int32_t n0 = i0 + kTokPerIter;
            np = load_raw<DT, VEC>(c.prow, n0, c.end);
            if (HASQ) nq = load_raw<DT, VEC>(c.qrow, n0, c.end);
        }
        // the workgroup's bound, possibly raised by another wavefront since the last iteration
        taup = fmaxf(taup, from_ordered_int(__hip_atomic_load(&lds.tau[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)));
        if (HASQ)
            tauq = fmaxf(tauq, from_ordered_int(__hip_atomic_load(&lds.tau[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)));
        const float taup_m = with_margin(taup);
        const float tauq_m = HASQ ? with_margin(tauq) : 0.0f;

        uint32_t x[8];
        philox4x32_10((uint32_t)i0 >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, x);
        philox4x32_10(((uint32_t)i0 >> 2) + 1, c.c1, c.c2, c.c3, a.key0, a.key1, x + 4);
        float lp[8], lq[8];
        unpack<RAWF32>(rp, lp);
        if (HASQ) unpack<RAWF32>(rq, lq);

        float accp = -INFINITY, accq = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float t = gumbel2_upper(x[e]);
            accp = fmaxf(accp, fmaf(lp[e], c2, t));
            if (HASQ) accq = fmaxf(accq, fmaf(lq[e], c2, t));
        }
        bool flag = accp >= taup_m;
        if (HASQ) flag = flag || (accq >= tauq_m);

        if (__builtin_amdgcn_ballot_w64(flag) != 0) {  // rare: some lane holds a token that may matter
            if (flag) {
#pragma unroll 1
                for (int e = 0; e < 8; ++e) {
                    const int32_t idx = i0 + e;
                    const float t = gumbel2_upper(x[e]);
                    const bool fp = fmaf(lp[e], c2, t) >= taup_m;
                    const bool fq = HASQ && (fmaf(lq[e], c2, t) >= tauq_m);
                    if ((fp || fq) && idx < c.end) {
                        const float l2e = log2_exponential(x[e]);
                        if (fp) refine_token(lp[e], l2e, c2, idx, taup, lds, 1);
                        if (fq) refine_token(lq[e], l2e, c2, idx, tauq, lds, 0);
                    }
                }
            }
            taup = wave_max(taup);
            if (HASQ) tauq = wave_max(tauq);
            if ((tid & (kWave - 1)) == 0) {
                atomicMax(&lds.tau[1], ordered_int(taup));
                if (HASQ) atomicMax(&lds.tau[0], ordered_int(tauq));
            }
        }
        rp = np;
        if (HASQ) rq = nq;
    }
    __syncthreads();

    // Exact stage: fp64 scores of the candidates, (score, lowest index) reduction, one partial per side.
#pragma unroll 1
    for (int side = HASQ ? 0 : 1; side < 2; ++side) {
        const char* row = side == 0 ? c.qrow : c.prow;
        const int32_t n = lds.count[side];
        if (n > kListCap) {  // workgroup-uniform: candidate list overflowed, score the whole split exactly
            exhaustive_side<DT>(a, c, row, side, lds.red_s, lds.red_i);
            continue;
        }
        double bs = -INFINITY;
        int32_t bi = -1;
        for (int32_t t = tid; t < n; t += kThreads) {
            const int32_t i = lds.list[side][t];
            const double s = exact_score_at(row, DT, i, a, c.c1, c.c2, c.c3);
            if (bi < 0 || better(s, i, bs, bi)) { bs = s; bi = i; }
        }
        block_argmax(bs, bi, lds.red_s, lds.red_i);
        if (tid == 0) {
            if (bi < 0) { bs = -INFINITY; bi = c.begin; }  // no finite score in this split
            store_partial(a, c, side, bs, bi);
        }
    }
}

template <int DT, bool VEC>
__global__ void __launch_bounds__(kThreads) race_filtered_kernel(RaceArgs a) {
    __shared__ Lds lds;
    const RowCtx c = make_ctx<DT>(a);
    if (c.qrow) race_filtered_body<DT, VEC, true>(a, c, lds);
    else race_filtered_body<DT, VEC, false>(a, c, lds);
}

// ------------------------------------------------------------------------------------------ finishing kernel
struct FinishArgs {
    const Partial* partials;
    int32_t nsplit;
    int32_t kd, kt, m;
    int32_t variant;
    const int32_t* parent;
    int32_t* draft_tokens;
    int32_t* target_tokens;
    int32_t* accept_len;
    int32_t* best_draft;
    int32_t* best_len;
    int32_t* accept_node;
};

__device__ __forceinline__ int32_t combine_partials(const Partial* p, int32_t nsplit) {
    double bs = p[0].score;
    int32_t bi = p[0].idx;
    for (int32_t s = 1; s < nsplit; ++s)
        if (p[s].score > bs) { bs = p[s].score; bi = p[s].idx; }  // splits are in index order: ties keep the lower
    return bi;
}

// One workgroup per prompt b: tokens of all its rows, then accept lengths.
__global__ void __launch_bounds__(kThreads) finish_kernel(FinishArgs f) {
    const int32_t b = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t seq0 = (int64_t)b * f.m;
    const int32_t nrows = f.m * f.kt;  // target rows of this prompt
    for (int32_t t = tid; t < nrows * 2; t += kThreads) {
        const int32_t side = t & 1, r = t >> 1;
        const int32_t d = r / f.kt, j = r % f.kt;
        const int64_t row = (seq0 + d) * f.kt + j;
        if (side == 0 && j >= f.kd) continue;
        const int32_t tok = combine_partials(f.partials + ((size_t)row * 2 + side) * f.nsplit, f.nsplit);
        if (side == 0) f.draft_tokens[(seq0 + d) * f.kd + j] = tok;
        else f.target_tokens[row] = tok;
    }
    __syncthreads();  // tokens of this prompt were written by this workgroup and are re-read below

    if (f.variant == ERSD_VARIANT_TREE) {
        // agree-path depth of every node by walking its ancestors (bounded by the node index)
        const int32_t N = f.kt;
        const int32_t* dt = f.draft_tokens + (int64_t)b * N;
        const int32_t* tt = f.target_tokens + (int64_t)b * N;
        int32_t best_depth = 0, best_node = -1;
        for (int32_t n = tid; n < N; n += kThreads) {
            int32_t depth = 0, cur = n;
            bool ok = true;
            while (true) {
                if (dt[cur] != tt[cur]) { ok = false; break; }
                ++depth;
                const int32_t p = f.parent[cur];
                if (p == -1) break;
                if (p < 0 || p >= cur) { ok = false; break; }  // malformed entry; p < cur bounds the walk
                cur = p;
            }
            if (ok && depth > best_depth) { best_depth = depth; best_node = n; }  // increasing n per thread
        }
        // reduce (depth desc, node asc)
        for (int off = kWave / 2; off > 0; off >>= 1) {
            const int32_t od = __shfl_xor(best_depth, off, kWave), on = __shfl_xor(best_node, off, kWave);
            if (od > best_depth || (od == best_depth && on >= 0 && (best_node < 0 || on < best_node))) {
                best_depth = od;
                best_node = on;
            }
        }
        __shared__ int32_t wd[kThreads / kWave], wn[kThreads / kWave];
        if ((tid & (kWave - 1)) == 0) { wd[tid / kWave] = best_depth; wn[tid / kWave] = best_node; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kThreads / kWave; ++w)
                if (wd[w] > best_depth || (wd[w] == best_depth && wn[w] >= 0 && (best_node < 0 || wn[w] < best_node))) {
                    best_depth = wd[w];
                    best_node = wn[w];
                }
            f.accept_len[b] = best_depth;
            if (f.accept_node) f.accept_node[b] = best_depth > 0 ? best_node : -1;
        }
        return;
    }

    // sequence / multi: first mismatch per draft
    for (int32_t d = tid; d < f.m; d += kThreads) {
        const int32_t* dt = f.draft_tokens + (seq0 + d) * f.kd;
        const int32_t* tt = f.target_tokens + (seq0 + d) * f.kt;
        int32_t acc = 0;
        while (acc < f.kd && dt[acc] == tt[acc]) ++acc;
        f.accept_len[seq0 + d] = acc;
    }
    if (f.best_len) {
        __syncthreads();
        if (tid == 0) {
            int32_t bl = -1, bd = -1;
            for (int32_t d = 0; d < f.m; ++d) {
                const int32_t v = f.accept_len[seq0 + d];
                if (v > bl) { bl = v; bd = d; }
            }
            f.best_len[b] = bl;
            f.best_draft[b] = bd;
        }
    }
}

// ------------------------------------------------------------------------------------------ self-check
// Checks, for every 32-bit word, the two fp32 facts the filter rests on against fp64:
//   gumbel2_upper(x) + kUpperSlack >= -log2 e(x)      and      |log2_exponential(x) - log2 e(x)| <= 2^-7.
__global__ void __launch_bounds__(kThreads) selftest_bounds_kernel(unsigned long long* counters) {
    unsigned long long bad_upper = 0, bad_refine = 0;
    float max_err = 0.0f, max_slack = 0.0f;
    const uint64_t stride = (uint64_t)gridDim.x * kThreads;
    for (uint64_t xi = (uint64_t)blockIdx.x * kThreads + threadIdx.x; xi < (1ull << 32); xi += stride) {
        const uint32_t x = (uint32_t)xi;
        const double v = ((double)x + 0.5) * 0x1p-32;
        const double truth = log2(-log1p(-v));  // log2 e
        const float up = gumbel2_upper(x) + kUpperSlack;
        if ((double)up < -truth) ++bad_upper;
        max_slack = fmaxf(max_slack, (float)((double)up + truth));
        const float err = fabsf((float)((double)log2_exponential(x) - truth));
        if (!(err <= 0x1p-7f)) ++bad_refine;
        max_err = fmaxf(max_err, err);
    }
    atomicAdd(&counters[0], bad_upper);
    atomicAdd(&counters[1], bad_refine);
    atomicMax(&counters[2], (unsigned long long)__float_as_uint(max_err));    // non-negative floats order as ints
    atomicMax(&counters[3], (unsigned long long)__float_as_uint(max_slack));
}

__global__ void zero_counters_kernel(unsigned long long* counters) {
    if (threadIdx.x < 4) counters[threadIdx.x] = 0;
}

// ------------------------------------------------------------------------------------------ host side
struct Plan {
    int32_t nsplit;
    int32_t chunk;
    int64_t rows;  // target rows = races
};

int env_int(const char* name, int dflt) {
    const char* s = std::getenv(name);
    if (!s || !*s) return dflt;
    return std::atoi(s);
}

// Split the vocabulary so that the grid has a few workgroups per SIMD even for few rows.
Plan make_plan(int64_t rows, int32_t V) {
    Plan p;
    p.rows = rows;
    const int64_t want_blocks = 256 * 8;  // 256 compute units
    int64_t ns = (want_blocks + rows - 1) / rows;
    const int64_t max_by_size = (V + 4 * kTokPerIter - 1) / (4 * kTokPerIter);  // at least 4 iterations per split
    if (ns > max_by_size) ns = max_by_size;
    const int forced = env_int("ERSD_FORCE_SPLIT", 0);  // tests only
    if (forced > 0) ns = forced;
    if (ns > kMaxSplit) ns = kMaxSplit;
    if (ns < 1) ns = 1;
    int64_t chunk = ((int64_t)V + ns - 1) / ns;
    chunk = (chunk + kTokPerIter - 1) / kTokPerIter * kTokPerIter;
    p.chunk = (int32_t)(chunk > 0x7fff0000LL ? 0x7fff0000LL : chunk);
    p.nsplit = (int32_t)(((int64_t)V + p.chunk - 1) / p.chunk);
    return p;
}

bool sizes_ok(int32_t B, int32_t m, int32_t kd, int32_t kt, int32_t V) {
    if (B < 1 || m < 1 || kd < 1 || kt < 1 || V < 1) return false;
    if (V > 0x7fff0000) return false;                       // token indices and split ends stay in int32
    const int64_t rows = (int64_t)B * m * kt;
    if (rows > (int64_t)0x7fffffff / kMaxSplit) return false;  // grid size and row counters stay in int32
    return true;
}

int check_common(const void* dl, const void* tl, ersd_dtype dt, float T, const void* ws) {
    if (!dl || !tl) return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (!(T > 0.0f) || !std::isfinite(T)) return ERSD_ERR_INVALID_ARG;
    if (((uintptr_t)dl & 15) || ((uintptr_t)tl & 15) || ((uintptr_t)ws & 15)) return ERSD_ERR_MISALIGNED;
    return ERSD_OK;
}

size_t workspace_for(const Plan& p) { return (size_t)p.rows * 2 * (size_t)p.nsplit * sizeof(Partial); }

struct Geometry {
    int32_t B, m, kd, kt, V;
};

// variant + public sizes -> rows per sequence; false if the sizes are not acceptable
bool geometry(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, Geometry& g) {
    if (k_or_N < 1 || k_or_N == 0x7fffffff) return false;
    g.B = B;
    g.V = V;
    if (variant == ERSD_VARIANT_SEQUENCE) { g.m = 1; g.kd = k_or_N; g.kt = k_or_N + 1; }
    else if (variant == ERSD_VARIANT_MULTI) { g.m = m; g.kd = k_or_N; g.kt = k_or_N + 1; }
    else if (variant == ERSD_VARIANT_TREE) { g.m = 1; g.kd = k_or_N; g.kt = k_or_N; }
    else return false;
    return sizes_ok(g.B, g.m, g.kd, g.kt, g.V);
}

int launch_races(const void* dl, const void* tl, ersd_dtype dt, const Geometry& g, float T, uint64_t seed, void* ws,
                 size_t ws_bytes, void* stream) {
    const Plan p = make_plan((int64_t)g.B * g.m * g.kt, g.V);
    if (ws_bytes < workspace_for(p)) return ERSD_ERR_WORKSPACE_TOO_SMALL;

    RaceArgs a;
    a.draft = static_cast<const char*>(dl);
    a.target = static_cast<const char*>(tl);
    a.partials = static_cast<Partial*>(ws);
    a.V = g.V;
    a.kd = g.kd;
    a.kt = g.kt;
    a.m = g.m;
    a.nsplit = p.nsplit;
    a.chunk = p.chunk;
    a.key0 = (uint32_t)(seed & 0xffffffffu);
    a.key1 = (uint32_t)(seed >> 32);
    a.T = (double)T;
    a.c2 = (float)(1.4426950408889634 / (double)T);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((uint32_t)(p.rows * p.nsplit)), block(kThreads);
    const bool vec = (g.V % 8) == 0;
    const char* mode = std::getenv("ERSD_KERNEL");  // tests only: "exhaustive" scores every token in fp64
    const bool exhaustive = mode && std::strcmp(mode, "exhaustive") == 0;
    if (exhaustive) {
        if (dt == ERSD_F32) hipLaunchKernelGGL(race_exhaustive_kernel<ERSD_F32>, grid, block, 0, s, a);
        else hipLaunchKernelGGL(race_exhaustive_kernel<ERSD_BF16>, grid, block, 0, s, a);
    } else if (dt == ERSD_F32) {
        if (vec) hipLaunchKernelGGL((race_filtered_kernel<ERSD_F32, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((race_filtered_kernel<ERSD_F32, false>), grid, block, 0, s, a);
    } else {
        if (vec) hipLaunchKernelGGL((race_filtered_kernel<ERSD_BF16, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((race_filtered_kernel<ERSD_BF16, false>), grid, block, 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int launch_finish(int variant, const Geometry& g, const int32_t* parent, int32_t* dtok, int32_t* ttok, int32_t* acc,
                  int32_t* best_draft, int32_t* best_len, int32_t* accept_node, const void* ws, size_t ws_bytes,
                  void* stream) {
    const Plan p = make_plan((int64_t)g.B * g.m * g.kt, g.V);
    if (ws_bytes < workspace_for(p)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    FinishArgs f;
    f.partials = static_cast<const Partial*>(ws);
    f.nsplit = p.nsplit;
    f.kd = g.kd;
    f.kt = g.kt;
    f.m = g.m;
    f.variant = variant;
    f.parent = parent;
    f.draft_tokens = dtok;
    f.target_tokens = ttok;
    f.accept_len = acc;
    f.best_draft = best_draft;
    f.best_len = best_len;
    f.accept_node = accept_node;
    hipLaunchKernelGGL(finish_kernel, dim3((uint32_t)g.B), dim3(kThreads), 0, static_cast<hipStream_t>(stream), f);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int launch(const void* dl, const void* tl, ersd_dtype dt, const Geometry& g, float T, uint64_t seed, int variant,
           const int32_t* parent, int32_t* dtok, int32_t* ttok, int32_t* acc, int32_t* best_draft, int32_t* best_len,
           int32_t* accept_node, void* ws, size_t ws_bytes, void* stream) {
    const int rc = launch_races(dl, tl, dt, g, T, seed, ws, ws_bytes, stream);
    if (rc != ERSD_OK) return rc;
    return launch_finish(variant, g, parent, dtok, ttok, acc, best_draft, best_len, accept_node, ws, ws_bytes, stream);
}

}  // namespace

extern "C" {

size_t ersd_race_workspace_bytes(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, ersd_dtype dt) {
    if (dt != ERSD_F32 && dt != ERSD_BF16) return 0;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return 0;
    return workspace_for(make_plan((int64_t)g.B * g.m * g.kt, g.V));
}

int ersd_race_stage_races(int variant, const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B,
                          int32_t m, int32_t k_or_N, int32_t V, float temperature, uint64_t seed, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (!workspace) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return ERSD_ERR_INVALID_ARG;
    return launch_races(draft_logits, target_logits, dt, g, temperature, seed, workspace, workspace_bytes, stream);
}

int ersd_race_stage_accept(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, const int32_t* parent,
                           int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len, int32_t* best_draft,
                           int32_t* best_len, int32_t* accept_node, const void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len || !workspace) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_TREE && !parent) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_MULTI && (!best_draft || !best_len)) return ERSD_ERR_NULL_POINTER;
    if ((uintptr_t)workspace & 15) return ERSD_ERR_MISALIGNED;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return ERSD_ERR_INVALID_ARG;
    if (variant != ERSD_VARIANT_MULTI) { best_draft = nullptr; best_len = nullptr; }
    if (variant != ERSD_VARIANT_TREE) { parent = nullptr; accept_node = nullptr; }
    return launch_finish(variant, g, parent, draft_tokens, target_tokens, accept_len, best_draft, best_len, accept_node,
                         workspace, workspace_bytes, stream);
}

int ersd_race_verify(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t k,
                     int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens, int32_t* target_tokens,
                     int32_t* accept_len, void* workspace, size_t workspace_bytes, void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len || !workspace) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(ERSD_VARIANT_SEQUENCE, B, 1, k, V, g)) return ERSD_ERR_INVALID_ARG;
    return launch(draft_logits, target_logits, dt, g, temperature, seed, ERSD_VARIANT_SEQUENCE, nullptr, draft_tokens,
                  target_tokens, accept_len, nullptr, nullptr, nullptr, workspace, workspace_bytes, stream);
}

int ersd_race_verify_multi(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t m,
                           int32_t k, int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens,
                           int32_t* target_tokens, int32_t* accept_len, int32_t* best_draft, int32_t* best_len,
                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len || !best_draft || !best_len || !workspace)
        return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(ERSD_VARIANT_MULTI, B, m, k, V, g)) return ERSD_ERR_INVALID_ARG;
    return launch(draft_logits, target_logits, dt, g, temperature, seed, ERSD_VARIANT_MULTI, nullptr, draft_tokens,
                  target_tokens, accept_len, best_draft, best_len, nullptr, workspace, workspace_bytes, stream);
}

int ersd_race_verify_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t N,
                          int32_t V, const int32_t* parent, float temperature, uint64_t seed, int32_t* draft_tokens,
                          int32_t* target_tokens, int32_t* accept_len, int32_t* accept_node, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (!parent || !draft_tokens || !target_tokens || !accept_len || !workspace) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(ERSD_VARIANT_TREE, B, 1, N, V, g)) return ERSD_ERR_INVALID_ARG;
    return launch(draft_logits, target_logits, dt, g, temperature, seed, ERSD_VARIANT_TREE, parent, draft_tokens,
                  target_tokens, accept_len, nullptr, nullptr, accept_node, workspace, workspace_bytes, stream);
}

int ersd_selftest_bounds(uint64_t* counters, void* stream) {
    if (!counters) return ERSD_ERR_NULL_POINTER;
    if ((uintptr_t)counters & 7) return ERSD_ERR_MISALIGNED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto* c = reinterpret_cast<unsigned long long*>(counters);
    hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, s, c);
    hipLaunchKernelGGL(selftest_bounds_kernel, dim3(256 * 16), dim3(kThreads), 0, s, c);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int ersd_tree_validate_host(const int32_t* parent_host, int32_t N) {
    if (!parent_host || N < 1) return 0;
    for (int32_t n = 0; n < N; ++n)
        if (parent_host[n] < -1 || parent_host[n] >= n) return 0;
    return 1;
}

const char* ersd_status_string(int status) {
    switch (status) {
        case ERSD_OK: return "ok";
        case ERSD_ERR_NULL_POINTER: return "null pointer argument";
        case ERSD_ERR_INVALID_ARG: return "invalid size or temperature";
        case ERSD_ERR_UNSUPPORTED_DTYPE: return "unsupported logit dtype";
        case ERSD_ERR_MISALIGNED: return "pointer not 16-byte aligned";
        case ERSD_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case ERSD_ERR_HIP: return "HIP kernel launch failed";
        default: return "unknown status";
    }
}

int ersd_version(void) { return 100; }

}  // extern "C"
