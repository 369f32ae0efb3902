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
//             of the row maximum.  (The comparison is made in units of 2^-23 with 159 taken off both
//             sides, so the bit pattern enters as it is; see tau_units.)
//   refine  : for those few tokens an fp32 score with a proven error margin, using v_log_f32; tokens
//             that can still be the maximum are appended to a candidate list in LDS and raise tau.
//   survive : when a row segment has been streamed, only candidates whose fp32 interval still reaches the
//             final tau survive (usually one); they are handed on as (index, logit, word) records.
//   exact   : the finishing kernel gathers a row's survivors from all its segments.  If one fp32 interval
//             lies above all others that token wins; otherwise the contenders are scored in fp64 exactly
//             as the definition says and reduced with the (score, lowest index) order.
//
// Since tau never exceeds the true row maximum and the bounds are one-sided, the true winner (and every
// token tied with it) is always among the survivors, so the result is the fp64 argmax.
//
// Work distribution: all rows are laid end to end in units of 8-token groups (a pair row weighs more than
// a target-only row) and cut into G equal shares, one per resident workgroup, so that every compute unit
// finishes at the same time whatever the shape.  A share is a list of row segments; each segment leaves
// its survivors per side in the workspace, and the finishing kernel resolves each row before it computes
// the accept lengths (first-mismatch scan, best draft, tree ancestor walk).

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <new>

#include "ersd.h"
#include "ersd_partition.h"
#include "ersd_philox.h"
#include "ersd_tree_plan.h"

namespace {

using namespace ersd_part;
using namespace ersd_philox;

#ifndef ERSD_THREADS
#define ERSD_THREADS 256
#endif
constexpr int kThreads = ERSD_THREADS;              // wavefronts per workgroup: kThreads / 64
#ifndef ERSD_STAGES
#define ERSD_STAGES 2
#endif
#ifndef ERSD_ROTATE_PRIO
#define ERSD_ROTATE_PRIO 2   // step of the priority rotation per tile; 0 switches it off
#endif
constexpr int kStages = ERSD_STAGES;                // register buffers per row: kStages - 1 tiles of loads in flight
constexpr int kListCap = 512;                       // candidate slots per side per workgroup
constexpr int kWave = 64;
constexpr int kWaves = kThreads / kWave;
constexpr uint32_t kMaxBlocks = 256 * 16;           // upper bound of resident workgroups, for workspace sizing

constexpr int kMaxSurvivors = 4;
constexpr int kMaxRank = ERSD_MAX_RANK;             // arrivals of one race a tree may use (Algorithm 5's child ranks)
constexpr int kMaxArrSurvivors = 16;                // survivors a segment hands on when the first arrivals are wanted
constexpr int32_t kMaxArrNodes = ERSD_MAX_ARRIVAL_TREE_NODES;

// What a row segment hands to the finishing kernel for one side: the tokens that can still be the row maximum.
struct Cand {
    int32_t idx;
    uint32_t word;   // the token's Philox word
    float logit;
    float s2;        // fp32 score in log2 units, error at most refine_err(s2)
};
struct SegOut {
    int32_t count;   // 0 = no finite score in the segment
    int32_t pad[3];
    Cand c[kMaxSurvivors];
};
struct SegOutArr {   // the same for a draft row of which the first arrivals (not only the winner) are wanted
    int32_t count;
    int32_t pad[3];
    Cand c[kMaxArrSurvivors];
};

struct RaceArgs {
    const char* draft;
    const char* target;
    SegOut* out;        // [row][side][slot]
    Part part;
    int32_t V;
    int64_t qstride, pstride;  // elements between the starts of consecutive draft / target rows (>= V)
    int32_t m;          // drafts per prompt
    uint64_t m_m;       // reciprocal of m (magic_of)
    uint32_t pos0;      // position index of a sequence's first row (counter word 1 = pos0 + j)
    uint32_t key0, key1;
    float c2;           // log2(e) / T
    int32_t exhaustive; // score every token in fp64 (reference path for tests)
    double T;
    // arrival trees only
    SegOutArr* outq;       // [row][slot]: draft-side survivors
    const int32_t* need;   // [kt]: arrivals wanted per context (0: the context has no child, its draft row is not read)
};

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

// (score, index) order: larger score first, then lower index.
__device__ __forceinline__ bool better(double s, int32_t i, double bs, int32_t bi) {
    return s > bs || (s == bs && i < bi);
}

__device__ __forceinline__ void wave_argmax(double& s, int32_t& i) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const double os = __shfl_xor(s, off, kWave);
        const int32_t oi = __shfl_xor(i, off, kWave);
        if (oi >= 0 && (i < 0 || better(os, oi, s, i))) { s = os; i = oi; }
    }
}

// One row segment handled by one workgroup.
struct Seg {
    const char* qrow;  // draft row or nullptr (bonus position)
    const char* prow;  // target row
    uint32_t c1, c2, c3;
    int32_t begin, end;  // token range, begin a multiple of 8
    uint64_t row;
    uint32_t slot;
    int32_t nq;          // arrival trees: arrivals wanted from the draft row (>= 1); 0 = only the winner, plain mode
};

struct Lds {
    float tau[2];        // the workgroup's lower bound of the row maximum, per side (raised with LDS float max)
    float tau_u[2];      // the same with its margin, in the filter's units: what the stream compares against
    int32_t count[2];    // candidates appended (may exceed kListCap: overflow)
    int32_t idx[2][kListCap];
    uint32_t word[2][kListCap];
    float logit[2][kListCap];
    int32_t nsurv[2];
    int32_t surv[2][kMaxArrSurvivors];  // list positions of the survivors
    double red_s[kWaves];
    int32_t red_i[kWaves];
    float top[kMaxRank];  // arrival trees: lower bounds of nq distinct draft-side tokens (see top_insert)
    int32_t rounds;       // arrival trees: exact selection rounds the segment's epilogue needs
};

// Exact scan of one side of a segment: every token scored in fp64.  The reference path, and the fallback when
// a candidate list overflows.  Waves 0-1 take side 0, waves 2-3 side 1 (lane best only; reduced by the caller).
// true iff (s, i) arrives after (ps, pi): smaller score, or the same score and a higher index
__device__ __forceinline__ bool arrives_after(double s, int32_t i, double ps, int32_t pi) {
    return s < ps || (s == ps && i > pi);
}

// The same restricted to the tokens that arrive after (ps, pi) and have a finite score: the next arrival.
template <int DT>
__device__ void exhaustive_half_after(const RaceArgs& a, const Seg& c, const char* row, int half_tid, bool has_prev,
                                      double ps, int32_t pi, double& bs, int32_t& bi) {
    const int32_t g0 = c.begin >> 2, g1 = (c.end + 3) >> 2;
    for (int32_t g = g0 + half_tid; g < g1; g += kThreads / 2) {
        uint32_t w[4];
        philox4x32((uint32_t)g, c.c1, c.c2, c.c3, a.key0, a.key1, w);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t i = g * 4 + e;
            if (i < c.end) {
                const double s = exact_score(widen_elem(row, DT, i), a.T, w[e]);
                if (!(s > -INFINITY) || (has_prev && !arrives_after(s, i, ps, pi))) continue;
                if (bi < 0 || s > bs) { bs = s; bi = i; }
            }
        }
    }
}

template <int DT>
__device__ void exhaustive_half(const RaceArgs& a, const Seg& c, const char* row, int half_tid, double& bs,
                                int32_t& bi) {
    const int32_t g0 = c.begin >> 2, g1 = (c.end + 3) >> 2;
    for (int32_t g = g0 + half_tid; g < g1; g += kThreads / 2) {
        uint32_t w[4];
        philox4x32((uint32_t)g, c.c1, c.c2, c.c3, a.key0, a.key1, w);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t i = g * 4 + e;
            if (i < c.end) {
                const double s = exact_score(widen_elem(row, DT, i), a.T, w[e]);
                if (bi < 0 || s > bs) { bs = s; bi = i; }  // increasing i per thread: ties keep the lower index
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ streaming filter
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct Raw {  // the two 16-byte pieces of a lane: bf16 -> 8 + 8 logits, fp32 -> 4 + 4
    u32x4 a, b;
};


// Geometry of a tile.  With 128-bit loads every lane takes two 16-byte pieces per row and tile, and the pieces
// are laid out so that each load instruction of a wavefront covers one contiguous kilobyte: lane t reads piece t
// and piece kThreads + t of the tile.
template <int DT>
struct TileShape {
    static constexpr int kTokPerPiece = DT == ERSD_BF16 ? 8 : 4;
    static constexpr int kTokPerThread = 2 * kTokPerPiece;
    static constexpr int kTile = kThreads * kTokPerThread;
    __device__ static __forceinline__ int32_t piece_a(int32_t tile_base, int tid) {
        return tile_base + tid * kTokPerPiece;
    }
    __device__ static __forceinline__ int32_t piece_b(int32_t tile_base, int tid) {
        return tile_base + (kThreads + tid) * kTokPerPiece;
    }
};

// The two pieces of one lane: tokens [ia, ia + kTokPerPiece) and [ib, ib + kTokPerPiece).
template <int DT>
__device__ __forceinline__ Raw load_raw(const char* row, int32_t ia, int32_t ib, int32_t end) {
    // Two unconditional 128-bit loads (no branch, so the compiler can count loads in flight exactly).  Piece starts
    // and `end` are multiples of the piece size and the segment is not empty; pieces past the end re-read the
    // segment's last piece instead, and the refine step never accepts a token index >= end.  A row starts wherever
    // the vocabulary size puts it, so the loads promise no more than element alignment (the hardware serves
    // unaligned 128-bit global loads; aligned rows lose nothing).
    // Byte offsets within a row fit 32 bits (the vocabulary is at most 2^30 tokens), so a load is the row's
    // address, which is the same for the whole wavefront, plus a 32-bit offset per lane: no 64-bit address arithmetic.
    typedef u32x4 u32x4_unaligned __attribute__((aligned(2)));
    constexpr uint32_t es = DT == ERSD_BF16 ? 2 : 4;
    const int32_t last = end - TileShape<DT>::kTokPerPiece;
    const uint32_t oa = (uint32_t)(ia < last ? ia : last) * es;
    const uint32_t ob = (uint32_t)(ib < last ? ib : last) * es;
    Raw r;
    r.a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_unaligned*>(row + oa));
    r.b = __builtin_nontemporal_load(reinterpret_cast<const u32x4_unaligned*>(row + ob));
    return r;
}

// Operands the hot loop wants in vector registers: on gfx950 the simple VALU operations issue faster when none of
// their sources is a scalar register or an inline constant, and the compiler would keep uniform values scalar.
struct HotConsts {
    float c2s;       // 2^23 * log2(e) / T: the logit's factor in the filter's fixed-point units (see bound_units)
    uint32_t sh16;   // the shift count 16
    uint32_t himask; // the upper half of a word: the odd element of a bf16 pair
};
__device__ __forceinline__ HotConsts make_hot_consts(float c2) {
    HotConsts h;
    const float c2s = c2 * 0x1p23f;
    asm volatile("v_mov_b32 %0, %1" : "=v"(h.c2s) : "s"(c2s));
    asm volatile("v_mov_b32 %0, 16" : "=v"(h.sh16));
    asm volatile("v_mov_b32 %0, 0xffff0000" : "=v"(h.himask));
    return h;
}

template <bool RAWF32>
__device__ __forceinline__ void unpack(const Raw& r, float l[8], uint32_t sh16) {
    if (RAWF32) {
        l[0] = __uint_as_float(r.a.x); l[1] = __uint_as_float(r.a.y);
        l[2] = __uint_as_float(r.a.z); l[3] = __uint_as_float(r.a.w);
        l[4] = __uint_as_float(r.b.x); l[5] = __uint_as_float(r.b.y);
        l[6] = __uint_as_float(r.b.z); l[7] = __uint_as_float(r.b.w);
    } else {
        const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            l[2 * e] = __uint_as_float(w[e] << sh16);
            l[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
    }
}

// The bit pattern of float(x), as a number: 2^23 * (127 + a piecewise-linear lower bound of log2 x).
__device__ __forceinline__ float bound_units(uint32_t x) {
    const float xf = (float)x;
    return (float)(int32_t)__float_as_uint(xf);
}
// Upper bound of -log2 e from the word x alone (see file header); slack is added to tau instead.
__device__ __forceinline__ float gumbel2_upper(uint32_t x) { return fmaf(bound_units(x), -0x1p-23f, 159.0f); }
// The filter compares in units of 2^-23 with 159 taken off both sides, which saves the scaling of every token's
// bound:  logit * c2 + gumbel2_upper(x) >= tau   <=>   logit * (2^23 c2) - bound_units(x) >= 2^23 (tau - 159).
// Values stay below 2^32 in magnitude for scores of ordinary size, so one rounding costs 2^-24 * 2^9 log2 units,
// far inside the margin with_margin() leaves; |logit| / T must stay below 2^100 for the product to be finite.
__device__ __forceinline__ float tau_units(float tau_m) { return fmaf(tau_m, 0x1p23f, -159.0f * 0x1p23f); }

// log2 of e = -ln(1 - v) in fp32.  |error| <= 2^-9 (the library's self-test checks it on the device for every
// 32-bit word; measured maximum 0.00097); callers use kRefineErr = 2^-7, four times that.
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

constexpr float kRefineErr = 0x1p-7f;
constexpr float kRelErr = 0x1p-20f;
constexpr float kUpperSlack = 0x1p-10f;
constexpr float kTauInit = -3.0e38f;  // below every finite score; -inf scores never reach it

// error bound of an fp32 score s2 (log2 units) against the true score
__device__ __forceinline__ float refine_err(float s2) { return fmaf(fabsf(s2), kRelErr, kRefineErr); }

__device__ __forceinline__ float with_margin(float tau) { return tau - fmaf(fabsf(tau), kRelErr, kUpperSlack); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ float lds_tau(const Lds& lds, int side) {
    return __hip_atomic_load(&lds.tau[side], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// The threshold the stream compares a bound against.  Every value ever stored comes from a valid lower bound of the
// row maximum, so the largest of them is valid too.
__device__ __forceinline__ float lds_tau_units(const Lds& lds, int side) {
    return __hip_atomic_load(&lds.tau_u[side], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_tau_raise(Lds& lds, int side, float v) {
    __hip_atomic_fetch_max(&lds.tau[side], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_max(&lds.tau_u[side], tau_units(with_margin(v)), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Arrival trees, draft side: tau must stay below the nq-th largest score of the segment.  lds.top holds lower
// bounds of up to nq DISTINCT tokens: every token is refined at most once and a bound enters only here, so the
// smallest of nq entries is below the nq-th largest score.  The lanes of a wavefront take turns; other wavefronts
// may interleave, which can lose an entry or mix two states in one read, but every value read is still the bound
// of a distinct token, so the returned bound (kTauInit if none) is valid whatever the interleaving.
__device__ __forceinline__ float top_insert(Lds& lds, int32_t nq, float lb) {
    float result = kTauInit;
    uint64_t todo = __builtin_amdgcn_ballot_w64(true);  // the lanes that are here
    const int lane = threadIdx.x & (kWave - 1);
    while (todo) {
        const int leader = __builtin_ctzll(todo);
        todo &= todo - 1;
        if (lane == leader) {
            float v[kMaxRank];
            float m = INFINITY;
            int am = 0;
#pragma unroll
            for (int r = 0; r < kMaxRank; ++r) {
                v[r] = r < nq ? __hip_atomic_load(&lds.top[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : INFINITY;
                if (v[r] < m) { m = v[r]; am = r; }
            }
            if (lb > m) {  // replaces the smallest entry (false for a NaN bound)
                __hip_atomic_store(&lds.top[am], lb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                float m2 = lb;
#pragma unroll
                for (int r = 0; r < kMaxRank; ++r)
                    if (r != am) m2 = fminf(m2, v[r]);
                result = m2;
            }
        }
    }
    return result;
}

// One side's refine step for one token of one lane.  nq > 0: the nq first arrivals are wanted, not only the winner.
__device__ __forceinline__ void refine_token(float logit, uint32_t x, float l2e, float c2, int32_t idx, float& tau,
                                             Lds& lds, int side, int32_t nq) {
    const float s2 = fmaf(logit, c2, -l2e);
    const float err = refine_err(s2);
    if (s2 > -INFINITY && s2 + err >= tau) {
        const int32_t pos = atomicAdd(&lds.count[side], 1);
        if (pos < kListCap) {
            lds.idx[side][pos] = idx;
            lds.word[side][pos] = x;
            lds.logit[side][pos] = logit;
        }
        tau = fmaxf(tau, nq > 0 ? top_insert(lds, nq, s2 - err) : s2 - err);
    }
}

// Element e (a run-time, wavefront-uniform index) of a lane's registers, by selects: keeps the rare refine loop
// rolled up and the arrays in registers.
__device__ __forceinline__ uint32_t pick4(const u32x4& v, int e) {
    uint32_t r = v.x;
    r = e == 1 ? v.y : r;
    r = e == 2 ? v.z : r;
    r = e == 3 ? v.w : r;
    return r;
}
template <bool RAWF32>
__device__ __forceinline__ float raw_logit(const Raw& r, int e) {
    if (RAWF32) return __uint_as_float(e < 4 ? pick4(r.a, e) : pick4(r.b, e - 4));
    const uint32_t w = pick4(r.a, e >> 1);
    return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
}

// the same with a compile-time index: a plain register reference
template <bool RAWF32>
__device__ __forceinline__ float raw_logit_const(const Raw& r, int e) {
    if (RAWF32) return __uint_as_float(e < 4 ? r.a[e & 3] : r.b[e & 3]);
    const uint32_t w = r.a[(e >> 1) & 3];
    return __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
}

// The rare second look at a lane's 8 tokens: those whose upper bound reaches tau get an fp32 score with an error
// margin; what can still be the maximum goes to the candidate list and raises tau (lane, wavefront, workgroup).
template <bool RAWF32, bool HASQ>
__device__ __forceinline__ void refine_tile(Lds& lds, float c2, int32_t i0, int32_t i1, int32_t end, const Raw& rq,
                                            const Raw& rp, const uint32_t (&x)[8], const float (&up)[8],
                                            const float (&uq)[8], bool flag, float tauq_u, float taup_u, int32_t nq) {
    if (!flag) return;
    float taup = lds_tau(lds, 1), tauq = HASQ ? lds_tau(lds, 0) : kTauInit;
    // which of this lane's (token, side) bounds reach tau: bits 0-7 target side, 8-15 draft side
    uint32_t mask = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (up[e] > taup_u) mask |= 1u << e;
        if (HASQ && uq[e] > tauq_u) mask |= 1u << (8 + e);
    }
    const float taup0 = taup, tauq0 = tauq;
    while (mask) {  // usually a single bit in a single lane
        const int b = __builtin_ctz(mask);
        mask &= mask - 1;
        const int e = b & 7;
        const bool isq = HASQ && b >= 8;
        const int32_t idx = e < 4 ? i0 + e : i1 + e - 4;
        if (idx < end) {
            const uint32_t xe = e < 4 ? pick4(u32x4{x[0], x[1], x[2], x[3]}, e) : pick4(u32x4{x[4], x[5], x[6], x[7]}, e - 4);
            const float lq = HASQ ? raw_logit<RAWF32>(rq, e) : 0.0f;
            const float lp = raw_logit<RAWF32>(rp, e);
            float tau = isq ? tauq : taup;
            refine_token(isq ? lq : lp, xe, log2_exponential(xe), c2, idx, tau, lds, isq ? 0 : 1, isq ? nq : 0);
            if (isq) tauq = tau;
            else taup = tau;
        }
    }
    // publish what this lane learned; the other lanes merge it in at their next tile
    if (taup > taup0) lds_tau_raise(lds, 1, taup);
    if (HASQ && tauq > tauq0) lds_tau_raise(lds, 0, tauq);
}

// The largest of the 8 logits a lane holds for one row of a tile, without widening them one by one.
//   fp32: a tree of three-input maxima.
//   bf16: the ordering of finite values of any IEEE-style format is the ordering of their sign-magnitude bit
//         patterns, so the packed half-precision maximum orders bf16 pairs correctly as long as no pattern reads
//         as a half-precision NaN (top five exponent bits set: |value| >= 2^121, infinities, NaN).  A -inf logit
//         (a masked token) reads as a quiet NaN, which the instruction drops in favour of the other operand, and
//         if all four operands of one half are masked the result is either -inf again or a NaN pattern that reads
//         as a huge bf16, which only sends the lane to the per-token bounds below.  The library's self-test checks
//         the instruction against the fp32 comparison for every pair of in-domain bf16 patterns.
// The instructions are written out because the compiler would first quiet possible signalling NaNs of loaded
// values, one more instruction per operand.
template <bool RAWF32>
__device__ __forceinline__ float group_max(const Raw& r, uint32_t himask, uint32_t sh16) {
    float m;
    if (RAWF32) {
        float m0, m1, m2;
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m0) : "v"(r.a.x), "v"(r.a.y), "v"(r.a.z));
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m1) : "v"(r.a.w), "v"(r.b.x), "v"(r.b.y));
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m2) : "v"(r.b.z), "v"(r.b.w), "v"(m0));
        asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(m1), "v"(m2));
    } else {
        uint32_t m01, m23, m4;
        asm("v_pk_max_f16 %0, %1, %2" : "=v"(m01) : "v"(r.a.x), "v"(r.a.y));
        asm("v_pk_max_f16 %0, %1, %2" : "=v"(m23) : "v"(r.a.z), "v"(r.a.w));
        asm("v_pk_max_f16 %0, %1, %2" : "=v"(m4) : "v"(m01), "v"(m23));
        const uint32_t hi = m4 & himask, lo = m4 << sh16;
        asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(hi), "v"(lo));
    }
    return m;
}

// The per-iteration work of one lane: 8 tokens of one or two rows.
template <bool RAWF32, bool HASQ, bool ARR>
__device__ __forceinline__ void filter_tile(const RaceArgs& a, const Seg& c, Lds& lds, const HotConsts& h, int32_t i0,
                                            int32_t i1, const Raw& rq, const Raw& rp, float tauq_u, float taup_u) {
    // tauq_u / taup_u: tau with its margin, in the filter's units.  The comparisons are strict, so a bound of -inf
    // (a masked token) never passes, not even while tau is still at its start value (-inf in these units).
    const float c2s = h.c2s;

    uint32_t x[8];
    philox4x32((uint32_t)i0 >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, x);      // tokens i0 .. i0 + 3
    philox4x32((uint32_t)i1 >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, x + 4);  // tokens i1 .. i1 + 3

    // One bound for the whole group first: the largest logit with the smallest word.  The word's term is
    // non-increasing in the word and the logit's factor is positive, and conversions and the fused multiply-add
    // round monotonically, so this is at least every token's own bound: if it stays below tau, so do all eight.
    const uint32_t xmin = min(min(min(x[0], x[1]), min(x[2], x[3])), min(min(x[4], x[5]), min(x[6], x[7])));
    const float tmin = bound_units(xmin);
    // (the two tests are combined without a short cut: a branch would cost more than the second bound)
    const bool gp = fmaf(group_max<RAWF32>(rp, h.himask, h.sh16), c2s, -tmin) > taup_u;
    const bool gq = HASQ ? fmaf(group_max<RAWF32>(rq, h.himask, h.sh16), c2s, -tmin) > tauq_u : false;
    const bool gflag = gp | gq;

    if (__builtin_amdgcn_ballot_w64(gflag) != 0) {  // some lane holds a group that may matter: token by token
        float lp[8], lq[8];
        unpack<RAWF32>(rp, lp, h.sh16);
        if (HASQ) unpack<RAWF32>(rq, lq, h.sh16);
        float accp = -INFINITY, accq = -INFINITY;
        float up[8], uq[8];  // per-token upper bounds of the two scores, in the filter's units
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float t = bound_units(x[e]);
            up[e] = fmaf(lp[e], c2s, -t);
            accp = fmaxf(accp, up[e]);
            if (HASQ) {
                uq[e] = fmaf(lq[e], c2s, -t);
                accq = fmaxf(accq, uq[e]);
            }
        }
        bool flag = accp > taup_u;
        if (HASQ) flag = flag || (accq > tauq_u);
        if (__builtin_amdgcn_ballot_w64(flag) != 0)  // rarer still: some token's own bound reaches tau
            refine_tile<RAWF32, HASQ>(lds, a.c2, i0, i1, c.end, rq, rp, x, up, uq, flag, tauq_u, taup_u,
                                      ARR ? c.nq : 0);
    }
}

// One lane's share of a tile: its two pieces.  A bf16 piece is 8 tokens and is filtered on its own; two fp32
// pieces make one group of 8.
template <int DT, bool HASQ, bool ARR>
__device__ __forceinline__ void filter_lane(const RaceArgs& a, const Seg& c, Lds& lds, const HotConsts& h, int32_t ia,
                                            int32_t ib, const Raw& rq, const Raw& rp) {
    constexpr bool RAWF32 = DT == ERSD_F32;
    // The workgroup's thresholds as they stand now: every lane publishes what it learns (refine_tile), so the
    // value in LDS is at least this lane's own and nothing is kept in registers from tile to tile.
    const float taup_u = lds_tau_units(lds, 1);
    const float tauq_u = HASQ ? lds_tau_units(lds, 0) : 0.0f;
    if (DT == ERSD_BF16) {
        Raw hq, hp;
        hq.a = rq.a; hq.b = rq.a; hp.a = rp.a; hp.b = rp.a;
        filter_tile<RAWF32, HASQ, ARR>(a, c, lds, h, ia, ia + 4, hq, hp, tauq_u, taup_u);
        hq.a = rq.b; hq.b = rq.b; hp.a = rp.b; hp.b = rp.b;
        filter_tile<RAWF32, HASQ, ARR>(a, c, lds, h, ib, ib + 4, hq, hp, tauq_u, taup_u);
    } else {
        filter_tile<RAWF32, HASQ, ARR>(a, c, lds, h, ia, ib, rq, rp, tauq_u, taup_u);
    }
}

// The n-th largest of the wavefront's 128 values (two per lane; kTauInit stands for "none"), by n rounds of
// maximum and knock-out.  All lanes of the wavefront call this.
__device__ __forceinline__ float wave_nth_largest(float v0, float v1, int32_t n) {
    float hi = fmaxf(v0, v1), lo = fminf(v0, v1), m = kTauInit;
    const int lane = threadIdx.x & (kWave - 1);
    for (int32_t r = 0; r < n; ++r) {
        m = wave_max(hi);
        const uint64_t holders = __builtin_amdgcn_ballot_w64(hi == m);
        if (lane == __builtin_ctzll(holders)) { hi = lo; lo = kTauInit; }
    }
    return m;
}

// The stream over a token range whose end is a multiple of 8.
template <int DT, bool HASQ, bool ARR>
__device__ void filter_stream(const RaceArgs& a, const Seg& c, Lds& lds) {
    constexpr bool RAWF32 = DT == ERSD_F32;
    typedef TileShape<DT> TS;
    constexpr int kTile = TS::kTile;
    const int tid = threadIdx.x;
    const float c2 = a.c2;

    // The loads of the first kStages - 1 tiles go out before anything else (the bootstrap below reads the first).
    // Memory latency is several microseconds under load while one wavefront filters a tile in well under one, so
    // every wavefront keeps kStages - 1 tiles in flight in a ring of register buffers.
    Raw q[kStages], pr[kStages];
    const int32_t first = TS::piece_a(c.begin, tid);
#pragma unroll
    for (int st = 0; st < kStages - 1; ++st) {
        const int32_t tb = c.begin + st * kTile;
        pr[st] = load_raw<DT>(c.prow, TS::piece_a(tb, tid), TS::piece_b(tb, tid), c.end);
        if (HASQ) q[st] = load_raw<DT>(c.qrow, TS::piece_a(tb, tid), TS::piece_b(tb, tid), c.end);
    }
    const Raw& pa = pr[0];
    const Raw& qa = q[0];

    // Bootstrap: each wavefront starts from a lower bound of the maximum: every lane scores, per side, the token
    // with the largest logit among the 8 it holds of the first tile (one logarithm per lane and side), and the
    // wavefront takes the best.  The better this start, the fewer group bounds reach tau while it is still rising.
    // (No barrier: the workgroup's bound in LDS is read at every tile.)
    {
        const int32_t i0 = first, i1 = RAWF32 ? TS::piece_b(c.begin, tid) : first + 4;
        uint32_t x[8];
        philox4x32((uint32_t)i0 >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, x);
        philox4x32((uint32_t)i1 >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, x + 4);
        float blp = -INFINITY, blq = -INFINITY;  // the lane's largest logit per side, and that token's word
        uint32_t bxp = 0, bxq = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int32_t idx = e < 4 ? i0 + e : i1 + e - 4;
            const bool in = idx < c.end;
            const float lp = raw_logit_const<RAWF32>(pa, e);
            if (in && lp > blp) { blp = lp; bxp = x[e]; }
            if (HASQ) {
                const float lq = raw_logit_const<RAWF32>(qa, e);
                if (in && lq > blq) { blq = lq; bxq = x[e]; }
            }
        }
        float taup = kTauInit, tauq = kTauInit;
        const float sp = fmaf(blp, c2, -log2_exponential(bxp));
        if (sp > -INFINITY) taup = sp - refine_err(sp);
        taup = wave_max(taup);
        if (HASQ) {
            const float sq = fmaf(blq, c2, -log2_exponential(bxq));
            float bq = kTauInit;
            if (sq > -INFINITY) bq = fmaxf(kTauInit, sq - refine_err(sq));
            // draft side: the largest bound, or (arrival trees) the nq-th largest of the wavefront's 64 tokens, which
            // is below the nq-th largest score of the segment.  These tokens are not entered into lds.top: the stream
            // meets them again.
            tauq = ARR && c.nq > 1 ? wave_nth_largest(bq, kTauInit, c.nq) : wave_max(bq);
        }
        if ((tid & (kWave - 1)) == 0) {
            lds_tau_raise(lds, 1, taup);
            if (HASQ) lds_tau_raise(lds, 0, tauq);
        }
    }

    const HotConsts h = make_hot_consts(a.c2);
#if ERSD_ROTATE_PRIO
    // The hardware issues from the oldest wavefront of a SIMD first, so the resident workgroups of a compute unit
    // would finish one after the other and the last would run alone, too few wavefronts to hide latency.  The
    // wavefronts of a SIMD therefore take turns at three priority levels, one step per tile, starting from their
    // slot number within the SIMD (hardware id register, bits 3:0), which differs between them.
    uint32_t turn = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 4);
#endif
    // kStages tiles per trip; buffer indices are compile-time constants, so the ring stays in registers
    for (int32_t base = c.begin; base < c.end; base += kStages * kTile) {
        bool done = false;
#pragma unroll
        for (int st = 0; st < kStages; ++st) {
            if (!done) {
#if ERSD_ROTATE_PRIO
                {
                    const uint32_t pr3 = turn % 3;
                    if (pr3 == 0) __builtin_amdgcn_s_setprio(0);
                    else if (pr3 == 1) __builtin_amdgcn_s_setprio(1);
                    else __builtin_amdgcn_s_setprio(2);
                    turn += (ERSD_ROTATE_PRIO);
                }
#endif
                constexpr int kAhead = kStages - 1;
                const int nb = (st + kAhead) % kStages;  // buffer of the tile kAhead tiles ahead
                const int32_t nt = base + (st + kAhead) * kTile, ct = base + st * kTile;
                pr[nb] = load_raw<DT>(c.prow, TS::piece_a(nt, tid), TS::piece_b(nt, tid), c.end);
                if (HASQ) q[nb] = load_raw<DT>(c.qrow, TS::piece_a(nt, tid), TS::piece_b(nt, tid), c.end);
                filter_lane<DT, HASQ, ARR>(a, c, lds, h, TS::piece_a(ct, tid), TS::piece_b(ct, tid), q[st], pr[st]);
                done = base + (st + 1) * kTile >= c.end;  // workgroup-uniform
            }
        }
    }
#if ERSD_ROTATE_PRIO
    __builtin_amdgcn_s_setprio(0);
#endif
}

// One segment: the 128-bit stream over its whole groups of 8 tokens, then the few tokens of a ragged row end (a
// vocabulary size that is not a multiple of 8), which go straight to the refine step.
template <int DT, bool HASQ, bool ARR>
__device__ void filter_segment(const RaceArgs& a, const Seg& c, Lds& lds) {
    const int32_t vend = c.end & ~7;  // c.begin is a multiple of 8
    if (vend > c.begin) {
        Seg v = c;
        v.end = vend;
        filter_stream<DT, HASQ, ARR>(a, v, lds);
    }
    const int32_t i = vend + (int32_t)threadIdx.x;
    if (i < c.end) {  // at most seven lanes
        float taup = lds_tau(lds, 1), tauq = HASQ ? lds_tau(lds, 0) : kTauInit;
        uint32_t w[4];
        philox4x32((uint32_t)i >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, w);
        const uint32_t x = pick4(u32x4{w[0], w[1], w[2], w[3]}, i & 3);
        const float l2e = log2_exponential(x);
        const float taup0 = taup, tauq0 = tauq;
        refine_token(widen_elem(c.prow, DT, i), x, l2e, a.c2, i, taup, lds, 1, 0);
        if (taup > taup0) lds_tau_raise(lds, 1, taup);
        if (HASQ) {
            refine_token(widen_elem(c.qrow, DT, i), x, l2e, a.c2, i, tauq, lds, 0, ARR ? c.nq : 0);
            if (tauq > tauq0) lds_tau_raise(lds, 0, tauq);
        }
    }
}

// Barrier of a workgroup that orders its LDS traffic only.  __syncthreads() also waits for every global store the
// wavefront has issued to be acknowledged, which under a streaming load takes microseconds; the survivor records a
// segment writes are read by the finishing kernel, never by this one, so the race kernels need no such wait.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// fp32 score of a (logit, word) record, exactly as the refine step computes it
__device__ __forceinline__ float score2(float logit, uint32_t word, float c2) {
    return fmaf(logit, c2, -log2_exponential(word));
}

// A whole segment: stream, then hand the survivors of each side to the finishing kernel.
template <int DT>
__device__ void race_segment(const RaceArgs& a, const Seg& c, Lds& lds) {
    const int tid = threadIdx.x;
    if (tid < 2) {
        lds.tau[tid] = kTauInit;
        lds.tau_u[tid] = -INFINITY;
        lds.count[tid] = 0;
        lds.nsurv[tid] = 0;
    }
    lds_barrier();
    if (!a.exhaustive) {
        if (c.qrow) filter_segment<DT, true, false>(a, c, lds);
        else filter_segment<DT, false, false>(a, c, lds);
    }
    lds_barrier();

    // Wavefronts 0-1 take the draft side, 2-3 the target side.
    const int side = tid / (kThreads / 2);
    const int half_tid = tid % (kThreads / 2);
    const char* row = side == 0 ? c.qrow : c.prow;
    const int32_t n = row ? lds.count[side] : 0;
    const bool listed = row && !a.exhaustive && n <= kListCap;
    if (listed) {  // keep the candidates whose interval still reaches the final lower bound
        const float tau = lds_tau(lds, side);
        for (int32_t t = half_tid; t < n; t += kThreads / 2) {
            const float s2 = score2(lds.logit[side][t], lds.word[side][t], a.c2);
            if (s2 + refine_err(s2) >= tau) {
                const int32_t k = atomicAdd(&lds.nsurv[side], 1);
                if (k < kMaxSurvivors) lds.surv[side][k] = t;
            }
        }
    }
    lds_barrier();
    SegOut* out = row ? a.out + (c.row * 2 + side) * a.part.nslot + c.slot : nullptr;
    const int32_t ns = lds.nsurv[side];
    const bool common = listed && ns <= kMaxSurvivors;
    double bs = -INFINITY;
    int32_t bi = -1;
    if (common) {  // 0 (no finite score), 1 or a few survivors
        if (half_tid == 0) out->count = ns;
        if (half_tid < ns) {
            const int32_t t = lds.surv[side][half_tid];
            Cand k;
            k.idx = lds.idx[side][t];
            k.word = lds.word[side][t];
            k.logit = lds.logit[side][t];
            k.s2 = score2(k.logit, k.word, a.c2);
            out->c[half_tid] = k;
        }
    } else if (row) {
        // Rare: too many survivors, an overflowed candidate list, or the reference mode.  Score in fp64 here and
        // hand on the single exact winner.
        if (a.exhaustive || n > kListCap) {
            exhaustive_half<DT>(a, c, row, half_tid, bs, bi);
        } else {
            for (int32_t t = half_tid; t < n; t += kThreads / 2) {
                const int32_t i = lds.idx[side][t];
                const double s = exact_score(lds.logit[side][t], a.T, lds.word[side][t]);
                if (bi < 0 || better(s, i, bs, bi)) { bs = s; bi = i; }
            }
        }
        wave_argmax(bs, bi);
        if ((tid & (kWave - 1)) == 0) { lds.red_s[tid / kWave] = bs; lds.red_i[tid / kWave] = bi; }
    }
    lds_barrier();
    if (!common && row && half_tid == 0) {
        const int w0 = side * (kWaves / 2);
        bs = lds.red_s[w0];
        bi = lds.red_i[w0];
        for (int w = w0 + 1; w < w0 + kWaves / 2; ++w) {
            const double os = lds.red_s[w];
            const int32_t oi = lds.red_i[w];
            if (oi >= 0 && (bi < 0 || better(os, oi, bs, bi))) { bs = os; bi = oi; }
        }
        if (bi < 0 || !(bs > -INFINITY)) {
            out->count = 0;
        } else {
            uint32_t w[4];
            philox4x32((uint32_t)bi >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, w);
            Cand k;
            k.idx = bi;
            k.word = w[bi & 3];
            k.logit = widen_elem(row, DT, bi);
            k.s2 = score2(k.logit, k.word, a.c2);
            out->count = 1;
            out->c[0] = k;
        }
    }
}

#ifndef ERSD_WAVES_PER_EU
#define ERSD_WAVES_PER_EU 3
#endif

// Which share a workgroup takes.  The hardware deals workgroups out to the eight accelerator dies (XCDs) in turn,
// workgroup i to die i mod 8, while the kind of a share (how many row starts it holds, whether it lies in
// target-only rows) repeats with the rows of a sequence; share = workgroup index would hand a die the same few
// kinds of share over and over, and the dies with the heavier kinds finish microseconds after the others.  Die x
// takes a contiguous range of shares instead, which holds every kind in the proportion of the whole job.
__device__ __forceinline__ uint32_t xcd_share(uint32_t block, uint32_t G) {
    constexpr uint32_t kXcds = 8;
    const uint32_t x = block % kXcds, per = G / kXcds, extra = G % kXcds;
    return x * per + (x < extra ? x : extra) + block / kXcds;
}

template <int DT>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(ERSD_WAVES_PER_EU, 8)))
race_kernel(RaceArgs a) {
    __shared__ Lds lds;
    const Part& p = a.part;
    const uint32_t share = xcd_share(blockIdx.x, p.G);
    const PartPos first = part_start_pos(p, share), last = part_start_pos(p, share + 1);
    const size_t es = DT == ERSD_F32 ? 4 : 2;
    // (row, sequence, position, prompt, draft) of the first segment; later segments start at the next row's
    // first group, so they follow by counting up
    uint64_t row = first.row;
    uint32_t g0 = first.grp;
    uint64_t seq = first.seq;
    uint32_t j = first.j;
    uint32_t prompt = p.fast ? magic_div((uint32_t)seq, a.m_m) : (uint32_t)(seq / a.m);
    uint32_t d = (uint32_t)(seq - (uint64_t)prompt * a.m);
    while (row < last.row || (row == last.row && g0 < last.grp)) {  // one row segment per trip (workgroup-uniform)
        Seg c;
        c.row = row;
        const uint32_t g1 = row == last.row ? last.grp : p.V8;
        c.prow = a.target + (size_t)row * (size_t)a.pstride * es;
        c.qrow = j < p.kd ? a.draft + (size_t)(seq * p.kd + j) * (size_t)a.qstride * es : nullptr;
        c.c1 = a.pos0 + j;
        c.c2 = prompt;
        c.c3 = d;
        c.nq = 0;
        c.begin = (int32_t)(g0 * 8);
        const int64_t e = (int64_t)g1 * 8;
        c.end = e < a.V ? (int32_t)e : a.V;
        // a segment that starts at its row's first group is that row's first writer
        c.slot = g0 == 0 ? 0 : share - part_first_block(p, seq, j);
        race_segment<DT>(a, c, lds);
        g0 = 0;
        ++row;
        if (++j == p.kt) {
            j = 0;
            ++seq;
            if (++d == (uint32_t)a.m) { d = 0; ++prompt; }
        }
    }
}

// ------------------------------------------------------------------------------------------ arrival trees
// Algorithm 5: every context has one race; its children are the first arrivals under the draft model.  A segment
// of a draft row hands on every token that can be among the row's first nq arrivals (usually nq of them).

// Partition as the device sees it: with a weight table the totals are known on the device only.
__device__ __forceinline__ Part part_on_device(const Part& in) {
    Part p = in;
    if (p.wprefix) {
        p.Us = (uint64_t)p.wprefix[p.kt] * p.V8;
        p.U = p.Us * (p.rows / p.kt);
    }
    return p;
}

template <int DT>
__device__ void race_segment_arr(const RaceArgs& a, const Seg& c, Lds& lds) {
    const int tid = threadIdx.x;
    if (tid < 2) {
        lds.tau[tid] = kTauInit;
        lds.tau_u[tid] = -INFINITY;
        lds.count[tid] = 0;
        lds.nsurv[tid] = 0;
    }
    if (tid < kMaxRank) lds.top[tid] = kTauInit;
    if (tid == 0) lds.rounds = 0;
    lds_barrier();
    if (!a.exhaustive) {
        if (c.qrow) filter_segment<DT, true, true>(a, c, lds);
        else filter_segment<DT, false, true>(a, c, lds);
    }
    lds_barrier();

    // Wavefronts 0-1 take the draft side, 2-3 the target side.
    const int side = tid / (kThreads / 2);
    const int half_tid = tid % (kThreads / 2);
    const char* row = side == 0 ? c.qrow : c.prow;
    const int32_t n = row ? lds.count[side] : 0;
    const bool listed = row && !a.exhaustive && n <= kListCap;
    const int32_t cap = side == 0 ? kMaxArrSurvivors : kMaxSurvivors;
    if (listed) {  // keep the candidates whose interval still reaches the final lower bound
        const float tau = lds_tau(lds, side);
        for (int32_t t = half_tid; t < n; t += kThreads / 2) {
            const float s2 = score2(lds.logit[side][t], lds.word[side][t], a.c2);
            if (s2 + refine_err(s2) >= tau) {
                const int32_t k = atomicAdd(&lds.nsurv[side], 1);
                if (k < cap) lds.surv[side][k] = t;
            }
        }
    }
    lds_barrier();
    int32_t* out_count = nullptr;
    Cand* out_rec = nullptr;
    if (row) {
        if (side == 0) {
            SegOutArr* o = a.outq + c.row * a.part.nslot + c.slot;
            out_count = &o->count;
            out_rec = o->c;
        } else {
            SegOut* o = a.out + (c.row * 2 + 1) * a.part.nslot + c.slot;
            out_count = &o->count;
            out_rec = o->c;
        }
    }
    const int32_t ns = lds.nsurv[side];
    const bool common = listed && ns <= cap;
    // Rare: too many survivors, an overflowed list, or the reference mode.  Then the wanted arrivals of the segment
    // are selected exactly, one per round: the best fp64 score among the tokens after the previous pick.
    const int32_t my_rounds = (row && !common) ? (side == 0 ? c.nq : 1) : 0;
    if (half_tid == 0 && my_rounds > 0) atomicMax(&lds.rounds, my_rounds);
    if (common) {
        if (half_tid == 0) *out_count = ns;
        if (half_tid < ns) {
            const int32_t t = lds.surv[side][half_tid];
            Cand k;
            k.idx = lds.idx[side][t];
            k.word = lds.word[side][t];
            k.logit = lds.logit[side][t];
            k.s2 = score2(k.logit, k.word, a.c2);
            out_rec[half_tid] = k;
        }
    }
    lds_barrier();
    const int32_t rounds = lds.rounds;  // workgroup-uniform
    const bool from_list = !(a.exhaustive || n > kListCap);
    double ps = 0.0;
    int32_t pi = -1, picked = 0;
    bool alive = my_rounds > 0;
    for (int32_t r = 0; r < rounds; ++r) {
        const bool mine = alive && r < my_rounds;
        double bs = -INFINITY;
        int32_t bi = -1;
        if (mine) {
            if (from_list) {
                for (int32_t t = half_tid; t < n; t += kThreads / 2) {
                    const int32_t i = lds.idx[side][t];
                    const double sc = exact_score(lds.logit[side][t], a.T, lds.word[side][t]);
                    if (!(sc > -INFINITY) || (r > 0 && !arrives_after(sc, i, ps, pi))) continue;
                    if (bi < 0 || better(sc, i, bs, bi)) { bs = sc; bi = i; }
                }
            } else {
                exhaustive_half_after<DT>(a, c, row, half_tid, r > 0, ps, pi, bs, bi);
            }
            wave_argmax(bs, bi);
            if ((tid & (kWave - 1)) == 0) { lds.red_s[tid / kWave] = bs; lds.red_i[tid / kWave] = bi; }
        }
        lds_barrier();
        if (mine) {  // every thread of the half combines its side's wavefronts the same way
            const int w0 = side * (kWaves / 2);
            bs = lds.red_s[w0];
            bi = lds.red_i[w0];
            for (int w = w0 + 1; w < w0 + kWaves / 2; ++w) {
                const double os = lds.red_s[w];
                const int32_t oi = lds.red_i[w];
                if (oi >= 0 && (bi < 0 || better(os, oi, bs, bi))) { bs = os; bi = oi; }
            }
            if (bi < 0) {
                alive = false;  // no further token with a finite score
            } else {
                ps = bs;
                pi = bi;
                if (half_tid == 0) {
                    uint32_t w[4];
                    philox4x32((uint32_t)bi >> 2, c.c1, c.c2, c.c3, a.key0, a.key1, w);
                    Cand k;
                    k.idx = bi;
                    k.word = w[bi & 3];
                    k.logit = widen_elem(row, DT, bi);
                    k.s2 = score2(k.logit, k.word, a.c2);
                    out_rec[picked] = k;
                }
                ++picked;
            }
        }
        lds_barrier();
    }
    if (my_rounds > 0 && half_tid == 0) *out_count = picked;
}

template <int DT>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(ERSD_WAVES_PER_EU, 8)))
race_arrivals_kernel(RaceArgs a) {
    __shared__ Lds lds;
    const Part p = part_on_device(a.part);
    const PartPos first = part_start_pos(p, blockIdx.x), last = part_start_pos(p, blockIdx.x + 1);
    const size_t es = DT == ERSD_F32 ? 4 : 2;
    uint64_t row = first.row;
    uint32_t g0 = first.grp;
    uint64_t seq = first.seq;
    uint32_t j = first.j;  // context
    // (the first two tests never fail for a partition made by this library; they keep a damaged weight table from
    // taking the loads out of the tensors)
    while (row < p.rows && g0 < p.V8 &&
           (row < last.row || (row == last.row && g0 < last.grp))) {  // one row segment per trip (workgroup-uniform)
        Seg c;
        c.row = row;
        const uint32_t g1 = row == last.row && last.grp < p.V8 ? last.grp : p.V8;
        c.nq = a.need[j];
        c.prow = a.target + (size_t)row * (size_t)a.pstride * es;
        c.qrow = c.nq > 0 ? a.draft + (size_t)row * (size_t)a.qstride * es : nullptr;
        c.c1 = j;
        c.c2 = (uint32_t)seq;
        c.c3 = 0;
        c.begin = (int32_t)(g0 * 8);
        const int64_t e = (int64_t)g1 * 8;
        c.end = e < a.V ? (int32_t)e : a.V;
        c.slot = g0 == 0 ? 0 : blockIdx.x - part_first_block(p, seq, j);
        if (c.slot >= p.nslot) break;  // (never for a partition made by this library: keeps the records in the workspace)
        race_segment_arr<DT>(a, c, lds);
        g0 = 0;
        ++row;
        if (++j == p.kt) { j = 0; ++seq; }
    }
}

// Shape of a (parent, rank) tree, computed once per call by one workgroup: valid[N], need[C] (arrivals wanted per
// context), wprefix[C + 1] (partition weights), C = N + 1.
struct ArrMeta {
    int32_t* valid;
    int32_t* need;
    uint32_t* wprefix;
};

__global__ void __launch_bounds__(kThreads) arrival_meta_kernel(const int32_t* parent, const int32_t* rank, int32_t N,
                                                                ArrMeta m) {
    const int tid = threadIdx.x;
    const int32_t C = N + 1;
    // small trees (the usual case) are read once into LDS; the scans below then run on LDS
    constexpr int32_t kStaged = 2048;
    __shared__ int32_t sp[kStaged], sr[kStaged], sv[kStaged];
    const bool staged = N <= kStaged;
    if (staged) {
        for (int32_t n = tid; n < N; n += kThreads) { sp[n] = parent[n]; sr[n] = rank[n]; }
        __syncthreads();
    }
    // 1. own[n]: a node's own entries are in range and no earlier sibling in range asks for the same arrival
    for (int32_t n = tid; n < N; n += kThreads) {
        const int32_t pa = staged ? sp[n] : parent[n], rk = staged ? sr[n] : rank[n];
        const bool ok = pa >= -1 && pa < n && rk >= 0 && rk < kMaxRank;
        bool dup = false;
        if (ok) {
            if (staged) {
                for (int32_t o = 0; o < n; ++o) dup |= sp[o] == pa && sr[o] == rk && sp[o] < o;
            } else {
                for (int32_t o = 0; o < n; ++o) {
                    const int32_t po = parent[o];
                    dup |= po == pa && rank[o] == rk && po < o;
                }
            }
        }
        const int32_t own = ok && !dup ? 1 : 0;
        if (staged) sv[n] = own;
        else m.valid[n] = own;
    }
    for (int32_t c = tid; c < C; c += kThreads) m.need[c] = 0;
    __syncthreads();
    // 2. valid[n]: own[] holds for the node and every ancestor (parent < node bounds the walk).  The large-tree
    // path keeps own[] in m.valid and marks "own but not valid" as 2 until every thread has finished reading.
    for (int32_t n = tid; n < N; n += kThreads) {
        bool ok = (staged ? sv[n] : m.valid[n]) != 0;
        const bool own = ok;
        int32_t cur = n;
        while (ok) {
            const int32_t pa = staged ? sp[cur] : parent[cur];
            if (pa == -1) break;
            ok = (staged ? sv[pa] : m.valid[pa]) != 0;
            cur = pa;
        }
        if (ok) atomicMax(&m.need[(staged ? sp[n] : parent[n]) + 1], (staged ? sr[n] : rank[n]) + 1);
        if (staged) m.valid[n] = ok ? 1 : 0;
        else if (own && !ok) m.valid[n] = 2;
    }
    __syncthreads();
    if (!staged)
        for (int32_t n = tid; n < N; n += kThreads)
            if (m.valid[n] == 2) m.valid[n] = 0;
    // 3. weights: a context with a draft row costs as a pair row
    __shared__ uint32_t part_sum[kThreads];
    const int32_t per = (C + kThreads - 1) / kThreads;
    const int32_t c0 = tid * per, c1 = c0 + per < C ? c0 + per : C;
    __syncthreads();
    uint32_t sum = 0;
    // need[] was raised with device atomics: read it past the first-level cache
    auto weight = [&](int32_t c) {
        return __hip_atomic_load(&m.need[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > 0 ? kWPair : kWSingle;
    };
    for (int32_t c = c0; c < c1; ++c) sum += weight(c);
    part_sum[tid] = sum;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {  // inclusive scan of the per-thread sums
        const uint32_t add = tid >= off ? part_sum[tid - off] : 0;
        __syncthreads();
        part_sum[tid] += add;
        __syncthreads();
    }
    uint32_t before = part_sum[tid] - sum;
    for (int32_t c = c0; c < c1; ++c) {
        m.wprefix[c] = before;
        before += weight(c);
    }
    if (c1 == C && c0 < C) m.wprefix[C] = before;
}

__device__ int32_t resolve_row(const SegOut* o, uint32_t nslots, double T, bool active, int lane8);

struct ArrFinishArgs {
    const SegOut* out;       // target-side survivors
    const SegOutArr* outq;
    Part part;
    double T;
    ArrMeta meta;
    int32_t* arrivals;       // [B, C, kMaxRank]
    const int32_t* parent;
    const int32_t* rank;
    int32_t N;
    int32_t* draft_tokens;   // [B, N]
    int32_t* target_tokens;  // [B, C]
    uint32_t target_blocks;  // leading workgroups of the resolve kernel that take the target side
    int32_t* accept_len;
    int32_t* accept_node;
    int32_t* emitted;        // [B, C]
};

// The first need[c] arrivals of every draft row from what its segments handed on: one wavefront per row scores
// the candidates in fp64 and picks them off in order (score descending, index ascending).
__global__ void __launch_bounds__(kThreads) resolve_arrivals_kernel(ArrFinishArgs f) {
    const int lane = threadIdx.x & (kWave - 1);
    const Part p = part_on_device(f.part);
    if (blockIdx.x < f.target_blocks) {  // winners under the target model: eight lanes per row, as in the other variants
        const uint64_t trow = (uint64_t)blockIdx.x * (kThreads / 8) + (threadIdx.x >> 3);
        const bool active = trow < p.rows;
        const uint64_t r = active ? trow : 0;
        const uint32_t n = active ? part_row_slots(p, r) : 0;
        const int32_t tok = resolve_row(f.out + (r * 2 + 1) * p.nslot, n, f.T, active, threadIdx.x & 7);
        if (active && (threadIdx.x & 7) == 0) f.target_tokens[r] = tok;
        return;
    }
    const uint64_t row = (uint64_t)(blockIdx.x - f.target_blocks) * kWaves + threadIdx.x / kWave;
    if (row >= p.rows) return;  // whole wavefront
    const int32_t nq = f.meta.need[row % p.kt];
    int32_t* arr = f.arrivals + row * kMaxRank;
    if (nq == 0) {
        if (lane < kMaxRank) arr[lane] = -1;
        return;
    }
    const uint32_t nsl = part_row_slots(p, row);
    const SegOutArr* o = f.outq + row * p.nslot;
    const uint32_t total = nsl * kMaxArrSurvivors;
    constexpr int kKeep = 4;  // scores kept in registers per lane; a row with more candidates recomputes the rest
    double sc[kKeep];
    int32_t id[kKeep];
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
        const uint32_t t = lane + k * kWave;
        id[k] = -1;
        sc[k] = 0.0;
        if (t < total) {
            const SegOutArr& so = o[t / kMaxArrSurvivors];
            const int32_t e = (int32_t)(t % kMaxArrSurvivors);
            if (e < so.count) {
                id[k] = so.c[e].idx;
                sc[k] = exact_score(so.c[e].logit, f.T, so.c[e].word);
            }
        }
    }
    double ps = 0.0;
    int32_t pi = -1;
    for (int32_t r = 0; r < kMaxRank; ++r) {  // uniform trip count: the lanes meet in shuffles
        double bs = -INFINITY;
        int32_t bi = -1;
        if (r < nq) {
#pragma unroll
            for (int k = 0; k < kKeep; ++k)
                if (id[k] >= 0 && sc[k] > -INFINITY && (r == 0 || arrives_after(sc[k], id[k], ps, pi)) &&
                    (bi < 0 || better(sc[k], id[k], bs, bi))) {
                    bs = sc[k];
                    bi = id[k];
                }
            for (uint32_t t = lane + kKeep * kWave; t < total; t += kWave) {
                const SegOutArr& so = o[t / kMaxArrSurvivors];
                const int32_t e = (int32_t)(t % kMaxArrSurvivors);
                if (e < so.count) {
                    const double v = exact_score(so.c[e].logit, f.T, so.c[e].word);
                    const int32_t i = so.c[e].idx;
                    if (v > -INFINITY && (r == 0 || arrives_after(v, i, ps, pi)) && (bi < 0 || better(v, i, bs, bi))) {
                        bs = v;
                        bi = i;
                    }
                }
            }
        }
        wave_argmax(bs, bi);
        if (lane == 0) arr[r] = r < nq ? bi : -1;  // -1: fewer tokens with a finite score than arrivals wanted
        if (bi >= 0) { ps = bs; pi = bi; }
        else ps = -INFINITY, pi = 0x7fffffff;      // nothing is left after this
    }
}

// Per prompt: the drafted token of every node, then the verification walk of Algorithm 5.
__global__ void __launch_bounds__(kThreads) arrival_walk_kernel(ArrFinishArgs f) {
    const int tid = threadIdx.x;
    const int32_t b = blockIdx.x, N = f.N, C = N + 1;
    int32_t* dtok = f.draft_tokens + (int64_t)b * N;
    const int32_t* ttok = f.target_tokens + (int64_t)b * C;
    int32_t* emitted = f.emitted + (int64_t)b * C;
    for (int32_t n = tid; n < N; n += kThreads)
        dtok[n] = f.meta.valid[n] ? f.arrivals[((int64_t)b * C + f.parent[n] + 1) * kMaxRank + f.rank[n]] : -1;
    for (int32_t c = tid; c < C; c += kThreads) emitted[c] = -1;
    __shared__ int32_t match;
    if (tid == 0) match = 0x7fffffff;
    __syncthreads();  // this workgroup's writes to dtok are re-read below
    int32_t ctx = 0, len = 0, node = -1;
    while (true) {  // the context index grows with every step, so at most C trips
        const int32_t t = ttok[ctx];
        for (int32_t n = tid; n < N; n += kThreads)
            if (f.meta.valid[n] && f.parent[n] + 1 == ctx && dtok[n] == t) atomicMin(&match, n);
        __syncthreads();
        const int32_t next = match;
        __syncthreads();
        if (tid == 0) {
            emitted[len] = t;
            match = 0x7fffffff;
        }
        __syncthreads();
        if (next == 0x7fffffff) break;
        ++len;
        node = next;
        ctx = next + 1;
    }
    if (tid == 0) {
        f.accept_len[b] = len;
        f.accept_node[b] = node;
    }
}

// ------------------------------------------------------------------------------------------ finishing kernel
struct FinishArgs {
    const SegOut* out;
    double T;
    Part part;
    int32_t m;
    int32_t variant;
    const int32_t* parent;
    int32_t* draft_tokens;
    int32_t* target_tokens;
    int32_t* accept_len;
    int32_t* best_draft;
    int32_t* best_len;
    int32_t* accept_node;
};

// The winner of one row side from the survivors its segments left: decided by the fp32 intervals when one lies
// above all others, by fp64 scores (lowest index on ties) among the contenders otherwise.  Eight adjacent lanes
// work on one row side, each taking every eighth segment slot; every lane of the wavefront must call this
// (`active` false for lanes without work) because the lanes of a group meet in shuffles.
//
// A row rarely has more than eight segments: each lane reads its first slot's record once into registers (named
// fields, no indexed array: nothing goes to scratch memory) and visits it three times; further slots are read again.
struct MySlots {
    const SegOut* o;
    uint32_t nslots;
    int lane8;
    int32_t cnt;       // survivors in the lane's first slot, never more than a record holds whatever it says
    Cand c0, c1, c2, c3;

    __device__ __forceinline__ void load(const SegOut* o_, uint32_t nslots_, bool active, int lane8_) {
        o = o_;
        nslots = active ? nslots_ : 0;
        lane8 = lane8_;
        cnt = 0;
        c0 = c1 = c2 = c3 = Cand{};
        if ((uint32_t)lane8 < nslots) {
            const SegOut& so = o[lane8];
            cnt = so.count < kMaxSurvivors ? so.count : kMaxSurvivors;
            c0 = so.c[0]; c1 = so.c[1]; c2 = so.c[2]; c3 = so.c[3];  // what lies past the count is never looked at
        }
    }
    template <typename F>
    __device__ __forceinline__ void for_each(F&& f) const {
        if (cnt > 0) f(c0);
        if (cnt > 1) f(c1);
        if (cnt > 2) f(c2);
        if (cnt > 3) f(c3);
        for (uint32_t sl = lane8 + 8; sl < nslots; sl += 8) {
            const int32_t n = o[sl].count;
#pragma unroll
            for (int32_t k = 0; k < kMaxSurvivors; ++k)
                if (k < n) f(o[sl].c[k]);
        }
    }
};

__device__ int32_t resolve_row(const SegOut* o, uint32_t nslots, double T, bool active, int lane8) {
    MySlots my;
    my.load(o, nslots, active, lane8);
    float lstar = -INFINITY;
    int32_t total = 0;
    my.for_each([&](const Cand& cd) {
        lstar = fmaxf(lstar, cd.s2 - refine_err(cd.s2));
        ++total;
    });
#pragma unroll
    for (int off = 4; off > 0; off >>= 1) {
        lstar = fmaxf(lstar, __shfl_xor(lstar, off, 8));
        total += __shfl_xor(total, off, 8);
    }
    int32_t contenders = 0, only = -1;
    my.for_each([&](const Cand& cd) {
        if (cd.s2 + refine_err(cd.s2) >= lstar) {
            ++contenders;
            only = cd.idx;
        }
    });
#pragma unroll
    for (int off = 4; off > 0; off >>= 1) {
        contenders += __shfl_xor(contenders, off, 8);
        only = max(only, __shfl_xor(only, off, 8));
    }
    if (total == 0) return 0;  // every score of the row is -inf: lowest index
    if (contenders == 1) return only;  // uniform over the eight lanes
    double bs = -INFINITY;
    int32_t bi = -1;
    my.for_each([&](const Cand& cd) {  // fp32 cannot tell: score the contenders exactly
        if (cd.s2 + refine_err(cd.s2) >= lstar) {
            const double sc = exact_score(cd.logit, T, cd.word);
            if (bi < 0 || better(sc, cd.idx, bs, bi)) { bs = sc; bi = cd.idx; }
        }
    });
#pragma unroll
    for (int off = 4; off > 0; off >>= 1) {
        const double os = __shfl_xor(bs, off, 8);
        const int32_t oi = __shfl_xor(bi, off, 8);
        if (oi >= 0 && (bi < 0 || better(os, oi, bs, bi))) { bs = os; bi = oi; }
    }
    return bi;
}

// Tokens: every (row, side) pair is resolved by eight lanes; 32 pairs per workgroup.
__global__ void __launch_bounds__(kThreads) resolve_kernel(FinishArgs f) {
    const int tid = threadIdx.x;
    const Part p = part_on_device(f.part);
    const uint64_t item = (uint64_t)blockIdx.x * (kThreads / 8) + (tid >> 3);
    const uint64_t row = item >> 1;
    const int side = (int)(item & 1);
    const uint32_t j = (uint32_t)(row % p.kt);
    const bool active = row < p.rows && (side == 1 || j < p.kd);
    const uint64_t r = active ? row : 0;
    const uint32_t n = active ? part_row_slots(p, r) : 0;
    const int32_t tok = resolve_row(f.out + (r * 2 + side) * p.nslot, n, f.T, active, tid & 7);
    if (active && (tid & 7) == 0) {
        if (side == 1) f.target_tokens[r] = tok;
        else f.draft_tokens[(r / p.kt) * p.kd + j] = tok;
    }
}

constexpr int kFinishMaxThreads = 1024;        // workgroup size of the one-launch finishing kernel, at most
constexpr int kFinishMaxItems = 2 * (kFinishMaxThreads / 8);  // (row, side) pairs per prompt it takes: two passes

// Accept lengths of prompt b from its tokens (first disagreement per draft, best draft, or the tree walk).
// dtok / ttok: the prompt's own tokens, [m][kd] and [m][kt], in global memory or in LDS.  Called by a whole
// workgroup (of any size up to kFinishMaxThreads) after the tokens are visible to it.
__device__ void accept_prompt(const FinishArgs& f, int32_t b, const int32_t* dtok, const int32_t* ttok,
                              const int32_t* parent) {
    const int tid = threadIdx.x, nthreads = blockDim.x;
    const Part& p = f.part;
    const int32_t kt = (int32_t)p.kt, kd = (int32_t)p.kd;
    const int64_t seq0 = (int64_t)b * f.m;

    if (f.variant == ERSD_VARIANT_TREE) {
        // agree-path depth of every node by walking its ancestors (bounded by the node index)
        const int32_t N = kt;
        int32_t best_depth = 0, best_node = -1;
        for (int32_t n = tid; n < N; n += nthreads) {
            int32_t depth = 0, cur = n;
            bool ok = true;
            while (true) {
                if (dtok[cur] != ttok[cur]) { ok = false; break; }
                ++depth;
                const int32_t pa = parent[cur];
                if (pa == -1) break;
                if (pa < 0 || pa >= cur) { ok = false; break; }  // malformed entry; pa < cur bounds the walk
                cur = pa;
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
        __shared__ int32_t wd[kFinishMaxThreads / kWave], wn[kFinishMaxThreads / kWave];
        if ((tid & (kWave - 1)) == 0) { wd[tid / kWave] = best_depth; wn[tid / kWave] = best_node; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < (nthreads + kWave - 1) / kWave; ++w)
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
    __shared__ int32_t best_bits;  // best draft: (accept length << 16 | 0xffff - draft), the largest wins
    if (tid == 0) best_bits = -1;
    if (f.best_len) __syncthreads();
    for (int32_t d = tid; d < f.m; d += nthreads) {
        const int32_t* dt = dtok + (int64_t)d * kd;
        const int32_t* tt = ttok + (int64_t)d * kt;
        int32_t acc = 0;
        while (acc < kd && dt[acc] == tt[acc]) ++acc;
        f.accept_len[seq0 + d] = acc;
        // longest accepted draft, lowest draft index among equals; lengths and draft counts beyond 16 bits take
        // the sequential path below
        if (f.best_len && kd < 0x7fff && f.m <= 0xffff) atomicMax(&best_bits, (acc << 16) | (0xffff - d));
    }
    if (f.best_len) {
        __syncthreads();
        if (tid == 0) {
            int32_t bl = -1, bd = -1;
            if (kd < 0x7fff && f.m <= 0xffff) {
                bl = best_bits >> 16;
                bd = 0xffff - (best_bits & 0xffff);
            } else {
                for (int32_t d = 0; d < f.m; ++d) {
                    const int32_t* dt = dtok + (int64_t)d * kd;
                    const int32_t* tt = ttok + (int64_t)d * kt;
                    int32_t acc = 0;
                    while (acc < kd && dt[acc] == tt[acc]) ++acc;
                    if (acc > bl) { bl = acc; bd = d; }
                }
            }
            f.best_len[b] = bl;
            f.best_draft[b] = bd;
        }
    }
}

// Accept lengths: one workgroup per prompt b, reading the tokens the previous kernel wrote.
__global__ void __launch_bounds__(kThreads) accept_kernel(FinishArgs f) {
    const int32_t b = blockIdx.x;
    accept_prompt(f, b, f.draft_tokens + (int64_t)b * f.m * f.part.kd, f.target_tokens + (int64_t)b * f.m * f.part.kt,
                  f.parent);
}

// Both steps in one launch, for prompts with up to kFinishMaxItems (row, side) pairs: workgroup b resolves the rows
// of prompt b itself, eight lanes per pair, and keeps the tokens in LDS for the acceptance step, so that nothing it
// wrote to global memory has to come back.
__global__ void __launch_bounds__(kFinishMaxThreads) finish_kernel(FinishArgs f) {
    __shared__ int32_t dtok[kFinishMaxItems], ttok[kFinishMaxItems], parent[kFinishMaxItems / 2];
    const int32_t b = blockIdx.x;
    const int tid = threadIdx.x, per_pass = blockDim.x / 8;
    const Part& p = f.part;
    if (f.variant == ERSD_VARIANT_TREE)  // the walk follows parent links: from LDS, not one memory round trip per step
        for (uint32_t n = tid; n < p.kt; n += blockDim.x) parent[n] = f.parent[n];
    const uint32_t rows_b = (uint32_t)f.m * p.kt;  // target rows of one prompt
    const uint64_t row0 = (uint64_t)b * rows_b;
    const uint32_t nitems = rows_b * 2;
    for (uint32_t first = 0; first < nitems; first += per_pass) {  // uniform trip count: lanes meet in shuffles
        const uint32_t item = first + (tid >> 3);
        const uint32_t lrow = item >> 1;                 // row within the prompt
        const int side = (int)(item & 1);
        const uint32_t j = lrow % p.kt;
        const bool active = item < nitems && (side == 1 || j < p.kd);
        const uint64_t r = active ? row0 + lrow : row0;
        const uint32_t n = active ? part_row_slots(p, r) : 0;
        const int32_t tok = resolve_row(f.out + (r * 2 + side) * p.nslot, n, f.T, active, tid & 7);
        if (active && (tid & 7) == 0) {
            if (side == 1) {
                f.target_tokens[r] = tok;
                ttok[lrow] = tok;
            } else {
                const uint32_t at = (lrow / p.kt) * p.kd + j;
                f.draft_tokens[(row0 / p.kt) * p.kd + at] = tok;
                dtok[at] = tok;
            }
        }
    }
    lds_barrier();  // the acceptance step reads the tokens from LDS
    accept_prompt(f, b, dtok, ttok, parent);
}

// ------------------------------------------------------------------------------------------ self-check
// Checks, for every 32-bit word, the two fp32 facts the filter rests on against fp64:
//   gumbel2_upper(x) + kUpperSlack >= -log2 e(x)      and      |log2_exponential(x) - log2 e(x)| <= 2^-9.
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
        if (!(err <= 0x1p-9f)) ++bad_refine;
        max_err = fmaxf(max_err, err);
    }
    // The packed half-precision maximum as an order on bf16 bit patterns (group_max): every pair of patterns, one in
    // each half of a word, both either finite with |value| < 2^121 or -inf.  The result must not be below the larger
    // of the two values (it may be above it only in the all-masked case, where the per-token bounds take over).
    unsigned long long bad_pkmax = 0;
    for (uint64_t xi = (uint64_t)blockIdx.x * kThreads + threadIdx.x; xi < (1ull << 32); xi += stride) {
        const uint32_t pa = (uint32_t)xi >> 16, pb = (uint32_t)xi & 0xffffu;
        const bool in_a = ((pa >> 10) & 0x1f) != 0x1f || pa == 0xff80u, in_b = ((pb >> 10) & 0x1f) != 0x1f || pb == 0xff80u;
        if (!in_a || !in_b) continue;
        uint32_t m;
        asm volatile("v_pk_max_f16 %0, %1, %2" : "=v"(m) : "v"(pa), "v"(pb));   // low halves compared
        const float fa = __uint_as_float(pa << 16), fb = __uint_as_float(pb << 16);
        const float got = __uint_as_float(m << 16);
        if (!(got >= fmaxf(fa, fb))) ++bad_pkmax;
        uint32_t mh;
        asm volatile("v_pk_max_f16 %0, %1, %2" : "=v"(mh) : "v"(pa << 16), "v"(pb << 16));   // high halves compared
        if ((mh >> 16) != (m & 0xffffu)) ++bad_pkmax;   // both halves of the instruction behave alike
    }
    atomicAdd(&counters[4], bad_pkmax);
    atomicAdd(&counters[0], bad_upper);
    atomicAdd(&counters[1], bad_refine);
    atomicMax(&counters[2], (unsigned long long)__float_as_uint(max_err));    // non-negative floats order as ints
    atomicMax(&counters[3], (unsigned long long)__float_as_uint(max_slack));
}

// Reads two buffers once with the race kernel's loads and launch shape and nothing else: what the memory system
// delivers to a kernel of this shape, for the benchmark to print beside the race kernel's rate.
__global__ void __launch_bounds__(kThreads) read_probe_kernel(const u32x4* a, uint64_t na, const u32x4* b, uint64_t nb,
                                                              uint32_t* sink) {
    const uint64_t n = na + nb, per = (n + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x, hi = lo + per < n ? lo + per : n;
    u32x4 acc = {0, 0, 0, 0};
    constexpr int kUnroll = 4;
    uint64_t i = lo + threadIdx.x;
    for (; i + (kUnroll - 1) * kThreads < hi; i += (uint64_t)kUnroll * kThreads) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t t = i + (uint64_t)u * kThreads;
            v[u] = __builtin_nontemporal_load(t < na ? a + t : b + (t - na));
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u];
    }
    for (; i < hi; i += kThreads) acc ^= __builtin_nontemporal_load(i < na ? a + i : b + (i - na));
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;  // keeps the loads; practically never true
}

__global__ void zero_counters_kernel(unsigned long long* counters) {
    if (threadIdx.x < 5) counters[threadIdx.x] = 0;
}

// ------------------------------------------------------------------------------------------ host side
struct Geometry {
    int32_t B, m, kd, kt, V;
    int64_t qstride, pstride;  // row strides in elements; 0 stands for V (rows back to back)
};

// a row stride is acceptable if rows do not overlap and the last row's end stays addressable
bool stride_ok(int64_t stride, int32_t V, int64_t rows) {
    return stride >= V && stride <= ((int64_t)1 << 40) && rows <= ((int64_t)1 << 60) / stride;
}

// Test and tuning hooks (ersd_test_hooks_set); a production process never sets them and no call reads the
// environment.
std::atomic<int> g_hook_blocks{0};        // > 0: workgroup count of the race kernels instead of the resident count
std::atomic<int> g_hook_exhaustive{0};    // != 0: every token scored in fp64 (the reference path inside the kernels)
std::atomic<int> g_hook_seg_cost{-1};     // >= 0: cost units charged to a row start instead of the built-in figure

bool sizes_ok(int32_t B, int32_t m, int32_t kd, int32_t kt, int32_t V) {
    if (B < 1 || m < 1 || kd < 1 || kt < 1 || V < 1) return false;
    if (V > (1 << 30)) return false;                          // token indices in int32, byte offsets within a row in 32 bits
    const int64_t rows = (int64_t)B * m * kt;
    if (rows > 0x7fffffff) return false;                      // grids and row indices
    const int64_t v8 = ((int64_t)V + 7) / 8;
    if (rows > ((int64_t)1 << 46) / v8) return false;         // cost units times workgroups stay below 2^63
    if ((int64_t)B * m > 0x7fffffff) return false;            // sequence counters are 32-bit counter words
    return true;
}

// variant + public sizes -> rows per sequence; false if the sizes are not acceptable
bool geometry(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, Geometry& g) {
    if (k_or_N < 1 || k_or_N == 0x7fffffff) return false;
    g.B = B;
    g.V = V;
    g.qstride = g.pstride = 0;
    if (variant == ERSD_VARIANT_SEQUENCE) { g.m = 1; g.kd = k_or_N; g.kt = k_or_N + 1; }
    else if (variant == ERSD_VARIANT_MULTI) { g.m = m; g.kd = k_or_N; g.kt = k_or_N + 1; }
    else if (variant == ERSD_VARIANT_TREE) { g.m = 1; g.kd = k_or_N; g.kt = k_or_N; }
    else return false;
    return sizes_ok(g.B, g.m, g.kd, g.kt, g.V);
}

// What a workgroup pays for starting another row (measured on an MI355X: a share with two row segments runs 5 to 6
// us longer than a share with the same bytes in one), in cost units: 10 units are one 8-token group of a row pair,
// 32 bytes of bf16 or 64 of fp32, and a workgroup streams about 8.5 bytes per nanosecond when all are running.
constexpr uint32_t kSegCostBf16 = 32000, kSegCostF32 = 16000;

std::atomic<int> g_hook_align{-1};        // >= 0: groups a share's start is aligned to (a power of two)
uint32_t align_mask_for(ersd_dtype dt) {
    const int h = g_hook_align.load(std::memory_order_relaxed);
    uint32_t a = h > 0 ? (uint32_t)h : (dt == ERSD_BF16 ? 8u : 4u);
    if (h == 0) a = 1;
    while (a & (a - 1)) a &= a - 1;  // a power of two
    return a - 1;
}

uint32_t seg_cost_for(ersd_dtype dt) {
    const int h = g_hook_seg_cost.load(std::memory_order_relaxed);
    if (h >= 0) return (uint32_t)h;
    return dt == ERSD_BF16 ? kSegCostBf16 : kSegCostF32;
}

// Partition for `blocks` resident workgroups (fewer if the job is small), with `seg_cost` cost units charged to
// every row start (less where shares are short: a share is always longer than two such charges).
Part make_part(const Geometry& g, uint32_t blocks, uint32_t seg_cost, uint32_t align_mask) {
    Part p{};
    p.V8 = (uint32_t)(((int64_t)g.V + 7) / 8);
    p.kd = (uint32_t)g.kd;
    p.kt = (uint32_t)g.kt;
    p.rows = (uint64_t)g.B * g.m * g.kt;
    p.wprefix = nullptr;
    const uint64_t seqs = (uint64_t)g.B * g.m;
    const uint64_t plain = ((uint64_t)kWPair * p.kd + (uint64_t)kWSingle * (p.kt - p.kd)) * p.V8 * seqs;  // no charges
    uint64_t G = blocks;
    const uint64_t by_quota = plain / kMinQuota;
    if (G > by_quota) G = by_quota;
    if (G < 1) G = 1;
    p.G = (uint32_t)G;
    const uint64_t cap = plain / G / 2;
    p.S = (uint32_t)(seg_cost < cap ? seg_cost : cap);
    // Shares start on whole 128-byte lines of the rows (8 groups of bf16, 4 of fp32): a wavefront's kilobyte loads
    // then cover 8 lines instead of 9 in every segment that starts inside a row.
    p.amask = align_mask;
    p.Lp = p.S + kWPair * p.V8;
    p.Ls = p.S + kWSingle * p.V8;
    p.pair_units = (uint64_t)p.Lp * p.kd;
    p.Us = p.pair_units + (uint64_t)p.Ls * (p.kt - p.kd);
    p.U = p.Us * seqs;
    p.nslot = (uint32_t)((uint64_t)p.Lp * p.G / p.U) + 2;
    p.fast = p.U < ((uint64_t)1 << 32) && p.rows < ((uint64_t)1 << 32) && p.U / p.G > p.G ? 1 : 0;
    if (p.fast) {
        p.q = (uint32_t)(p.U / p.G);
        p.r = (uint32_t)(p.U % p.G);
        p.m_G = magic_of(p.G);
        p.m_q = magic_of(p.q);
        p.m_Us = magic_of(p.Us);
        p.m_pair_row = magic_of(p.Lp);
        p.m_single_row = magic_of(p.Ls);
        p.m_kt = magic_of(p.kt);
    }
    return p;
}

size_t workspace_for(const Geometry& g) {
    // slots per row grow with the workgroup count and are most when no row start is charged: size for that
    const Part p = make_part(g, kMaxBlocks, 0, 0);
    return (size_t)p.rows * 2 * p.nslot * sizeof(SegOut);
}

int check_common(const void* dl, const void* tl, ersd_dtype dt, float T, const void* ws) {
    if (!dl || !tl) return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (!(T > 0.0f) || !std::isfinite(T)) return ERSD_ERR_INVALID_ARG;
    if (((uintptr_t)dl & 15) || ((uintptr_t)tl & 15) || ((uintptr_t)ws & 15)) return ERSD_ERR_MISALIGNED;
    return ERSD_OK;
}

template <typename K>
int resident_blocks(K kernel, std::atomic<int>& cache) {
    int v = cache.load(std::memory_order_relaxed);
    if (v > 0) return v;
    int per_cu = 0, dev = 0;
    hipDeviceProp_t prop;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kThreads, 0) != hipSuccess || per_cu < 1 ||
        hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
        return -1;
    // Three workgroups per compute unit (one wavefront of each per SIMD) is the best count also where more would
    // fit: the fp32 kernel needs fewer registers and could hold four, which measured 2 % slower on the large fp32
    // workload.
    if (per_cu > ERSD_WAVES_PER_EU * (4 * kWave / kThreads)) per_cu = ERSD_WAVES_PER_EU * (4 * kWave / kThreads);
    v = per_cu * prop.multiProcessorCount;
    if (v > (int)kMaxBlocks) v = (int)kMaxBlocks;
    cache.store(v, std::memory_order_relaxed);
    return v;
}

// Workgroups the race kernel is launched with: as many as are resident at once on the current device.
int race_blocks(ersd_dtype dt) {
    static std::atomic<int> cache[2];
    const int forced = g_hook_blocks.load(std::memory_order_relaxed);
    if (forced > 0) return forced > (int)kMaxBlocks ? (int)kMaxBlocks : forced;
    return dt == ERSD_F32 ? resident_blocks(race_kernel<ERSD_F32>, cache[0])
                          : resident_blocks(race_kernel<ERSD_BF16>, cache[1]);
}

// The partition both stages use.  It depends on the device (resident workgroups), so both stages recompute it
// the same way; `nslot` is capped by what the workspace was sized for.
int plan_part(const Geometry& g, ersd_dtype dt, size_t ws_bytes, Part& p) {
    if (ws_bytes < workspace_for(g)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    const int blocks = race_blocks(dt);
    if (blocks < 1) return ERSD_ERR_HIP;
    p = make_part(g, (uint32_t)blocks, seg_cost_for(dt), align_mask_for(dt));
    if (ws_bytes < (size_t)p.rows * 2 * p.nslot * sizeof(SegOut)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    return ERSD_OK;
}

int launch_races(const void* dl, const void* tl, ersd_dtype dt, const Geometry& g, float T, uint64_t seed, void* ws,
                 size_t ws_bytes, void* stream, uint32_t pos0 = 0) {
    RaceArgs a{};
    const int rc = plan_part(g, dt, ws_bytes, a.part);
    if (rc != ERSD_OK) return rc;
    a.draft = static_cast<const char*>(dl);
    a.target = static_cast<const char*>(tl);
    a.out = static_cast<SegOut*>(ws);
    a.V = g.V;
    a.qstride = g.qstride ? g.qstride : g.V;
    a.pstride = g.pstride ? g.pstride : g.V;
    a.m = g.m;
    a.m_m = magic_of((uint64_t)g.m);
    a.pos0 = pos0;
    a.key0 = (uint32_t)(seed & 0xffffffffu);
    a.key1 = (uint32_t)(seed >> 32);
    a.T = (double)T;
    a.c2 = (float)(1.4426950408889634 / (double)T);
    a.exhaustive = g_hook_exhaustive.load(std::memory_order_relaxed) != 0;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(a.part.G), block(kThreads);
    if (dt == ERSD_F32) hipLaunchKernelGGL(race_kernel<ERSD_F32>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(race_kernel<ERSD_BF16>, grid, block, 0, s, a);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int launch_finish(int variant, const Geometry& g, ersd_dtype dt, float T, const int32_t* parent, int32_t* dtok,
                  int32_t* ttok,
                  int32_t* acc, int32_t* best_draft, int32_t* best_len, int32_t* accept_node, const void* ws,
                  size_t ws_bytes, void* stream) {
    FinishArgs f{};
    const int rc = plan_part(g, dt, ws_bytes, f.part);
    if (rc != ERSD_OK) return rc;
    f.out = static_cast<const SegOut*>(ws);
    f.T = (double)T;
    f.m = g.m;
    f.variant = variant;
    f.parent = parent;
    f.draft_tokens = dtok;
    f.target_tokens = ttok;
    f.accept_len = acc;
    f.best_draft = best_draft;
    f.best_len = best_len;
    f.accept_node = accept_node;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t items = f.part.rows * 2;
    if (variant < 0) {  // tokens only
        hipLaunchKernelGGL(resolve_kernel, dim3((uint32_t)((items + kThreads / 8 - 1) / (kThreads / 8))),
                           dim3(kThreads), 0, s, f);
    } else if ((uint64_t)g.m * g.kt * 2 <= (uint64_t)kFinishMaxItems) {  // at most two passes per prompt: one launch
        // eight lanes per (row, side) pair of a prompt, whole wavefronts, at most kFinishMaxThreads
        uint32_t threads = (uint32_t)g.m * g.kt * 2 * 8;
        threads = threads > (uint32_t)kFinishMaxThreads ? (uint32_t)kFinishMaxThreads : (threads + kWave - 1) / kWave * kWave;
        hipLaunchKernelGGL(finish_kernel, dim3((uint32_t)g.B), dim3(threads), 0, s, f);
    } else {
        hipLaunchKernelGGL(resolve_kernel, dim3((uint32_t)((items + kThreads / 8 - 1) / (kThreads / 8))),
                           dim3(kThreads), 0, s, f);
        hipLaunchKernelGGL(accept_kernel, dim3((uint32_t)g.B), dim3(kThreads), 0, s, f);
    }
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int launch(const void* dl, const void* tl, ersd_dtype dt, const Geometry& g, float T, uint64_t seed, int variant,
           const int32_t* parent, int32_t* dtok, int32_t* ttok, int32_t* acc, int32_t* best_draft, int32_t* best_len,
           int32_t* accept_node, void* ws, size_t ws_bytes, void* stream) {
    const int rc = launch_races(dl, tl, dt, g, T, seed, ws, ws_bytes, stream);
    if (rc != ERSD_OK) return rc;
    return launch_finish(variant, g, dt, T, parent, dtok, ttok, acc, best_draft, best_len, accept_node, ws, ws_bytes,
                         stream);
}

// ---- library-owned scratch memory for the entry point that allocates nothing
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only a
// stand-in for the symbol: the device address comes from hipGetSymbolAddress, asked once per device with that device
// current, and only that address is ever handed to a kernel.
constexpr size_t kScratchBytes = (size_t)ERSD_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ERSD_ERR_HIP;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return ERSD_ERR_HIP;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // every thread finds the same address
    }
    *out = ptr;
    return ERSD_OK;
}

// ---- arrival trees: sizes, workspace layout, launches
bool arrival_sizes_ok(int32_t B, int32_t N, int32_t V) {
    if (N < 1 || N > kMaxArrNodes) return false;
    return sizes_ok(B, 1, N + 1, N + 1, V);
}

uint32_t arrival_nslot(int32_t B, int32_t C, uint32_t G) {
    // a row has at most kWPair * V8 cost units and a share at least kWSingle * V8 * B * C / G of them
    return (uint32_t)(((uint64_t)kWPair * G) / ((uint64_t)kWSingle * B * C)) + 2;
}

uint32_t arrival_blocks(int32_t B, int32_t C, int32_t V, uint32_t blocks) {
    const uint64_t v8 = ((uint64_t)V + 7) / 8;
    uint64_t G = blocks;
    const uint64_t by_quota = (uint64_t)kWSingle * v8 * B * C / kMinQuota;
    if (G > by_quota) G = by_quota;
    return G < 1 ? 1u : (uint32_t)G;
}

struct ArrLayout {
    size_t out, outq, arrivals, valid, need, wprefix, total;
};

using ersd_plan::align16;
using ersd_plan::PlanLayout;
using ersd_plan::plan_layout;

ArrLayout arrival_layout(int32_t B, int32_t N, int32_t V) {
    const int32_t C = N + 1;
    const uint64_t rows = (uint64_t)B * C;
    const uint32_t nslot = arrival_nslot(B, C, arrival_blocks(B, C, V, kMaxBlocks));  // the most any launch uses
    ArrLayout l;
    l.out = 0;
    l.outq = align16(l.out + rows * 2 * nslot * sizeof(SegOut));
    l.arrivals = align16(l.outq + rows * nslot * sizeof(SegOutArr));
    l.valid = align16(l.arrivals + rows * kMaxRank * sizeof(int32_t));
    l.need = align16(l.valid + (size_t)N * sizeof(int32_t));
    l.wprefix = align16(l.need + (size_t)C * sizeof(int32_t));
    l.total = align16(l.wprefix + (size_t)(C + 1) * sizeof(uint32_t));
    return l;
}

// The partition of an arrival tree: every field is set here (the struct is value-initialised, `fast` stays 0: plain
// division, because the totals are known only where the weight table is), and the table's totals are filled in by
// part_on_device where the table can be read.
Part make_arrival_part(int32_t B, int32_t C, int32_t V, uint32_t blocks, const uint32_t* wprefix, ersd_dtype dt) {
    Part p{};
    p.amask = align_mask_for(dt);  // shares start on whole cache lines of the rows
    p.V8 = (uint32_t)(((int64_t)V + 7) / 8);
    p.kd = 0;                    // no closed-form pair rows: the table decides
    p.kt = (uint32_t)C;
    p.rows = (uint64_t)B * C;
    p.G = arrival_blocks(B, C, V, blocks);
    p.nslot = arrival_nslot(B, C, p.G);
    p.wprefix = wprefix;
    return p;
}

int arrival_race_blocks(ersd_dtype dt) {
    static std::atomic<int> cache[2];
    const int forced = g_hook_blocks.load(std::memory_order_relaxed);
    if (forced > 0) return forced > (int)kMaxBlocks ? (int)kMaxBlocks : forced;
    return dt == ERSD_F32 ? resident_blocks(race_arrivals_kernel<ERSD_F32>, cache[0])
                          : resident_blocks(race_arrivals_kernel<ERSD_BF16>, cache[1]);
}

int launch_arrival_tree(const void* dl, int64_t qstride, const void* tl, int64_t pstride, ersd_dtype dt, int32_t B,
                        int32_t N, int32_t V,
                        const int32_t* parent, const int32_t* rank, float T, uint64_t seed, int32_t* dtok,
                        int32_t* ttok, int32_t* acc, int32_t* accept_node, int32_t* emitted, void* ws, void* stream,
                        const void* plan = nullptr) {
    const int32_t C = N + 1;
    const int blocks = arrival_race_blocks(dt);
    if (blocks < 1) return ERSD_ERR_HIP;
    const ArrLayout l = arrival_layout(B, N, V);
    char* base = static_cast<char*>(ws);
    ArrMeta meta{};
    if (plan) {  // the tree's shape was derived earlier (ersd_arrival_tree_prepare): read only from here on
        const PlanLayout pl = plan_layout(N);
        char* pb = const_cast<char*>(static_cast<const char*>(plan));
        meta.valid = reinterpret_cast<int32_t*>(pb + pl.valid);
        meta.need = reinterpret_cast<int32_t*>(pb + pl.need);
        meta.wprefix = reinterpret_cast<uint32_t*>(pb + pl.wprefix);
    } else {
        meta.valid = reinterpret_cast<int32_t*>(base + l.valid);
        meta.need = reinterpret_cast<int32_t*>(base + l.need);
        meta.wprefix = reinterpret_cast<uint32_t*>(base + l.wprefix);
    }

    const Part p = make_arrival_part(B, C, V, (uint32_t)blocks, meta.wprefix, dt);

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!plan) hipLaunchKernelGGL(arrival_meta_kernel, dim3(1), dim3(kThreads), 0, s, parent, rank, N, meta);

    RaceArgs a{};
    a.draft = static_cast<const char*>(dl);
    a.target = static_cast<const char*>(tl);
    a.out = reinterpret_cast<SegOut*>(base + l.out);
    a.outq = reinterpret_cast<SegOutArr*>(base + l.outq);
    a.need = meta.need;
    a.part = p;
    a.V = V;
    a.qstride = qstride;
    a.pstride = pstride;
    a.m = 1;
    a.m_m = 0;
    a.pos0 = 0;
    a.key0 = (uint32_t)(seed & 0xffffffffu);
    a.key1 = (uint32_t)(seed >> 32);
    a.T = (double)T;
    a.c2 = (float)(1.4426950408889634 / (double)T);
    a.exhaustive = g_hook_exhaustive.load(std::memory_order_relaxed) != 0;
    const dim3 grid(p.G), block(kThreads);
    if (dt == ERSD_F32) hipLaunchKernelGGL(race_arrivals_kernel<ERSD_F32>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(race_arrivals_kernel<ERSD_BF16>, grid, block, 0, s, a);

    ArrFinishArgs af{};
    af.out = a.out;
    af.outq = a.outq;
    af.target_blocks = (uint32_t)((p.rows + kThreads / 8 - 1) / (kThreads / 8));
    af.part = p;
    af.T = (double)T;
    af.meta = meta;
    af.arrivals = reinterpret_cast<int32_t*>(base + l.arrivals);
    af.parent = parent;
    af.rank = rank;
    af.N = N;
    af.draft_tokens = dtok;
    af.target_tokens = ttok;
    af.accept_len = acc;
    af.accept_node = accept_node;
    af.emitted = emitted;
    hipLaunchKernelGGL(resolve_arrivals_kernel,
                       dim3(af.target_blocks + (uint32_t)((p.rows + kWaves - 1) / kWaves)), dim3(kThreads), 0, s, af);
    hipLaunchKernelGGL(arrival_walk_kernel, dim3((uint32_t)B), dim3(kThreads), 0, s, af);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

}  // namespace

extern "C" {

size_t ersd_race_arrival_tree_workspace_bytes(int32_t B, int32_t N, int32_t V, ersd_dtype dt) {
    if (dt != ERSD_F32 && dt != ERSD_BF16) return 0;
    if (!arrival_sizes_ok(B, N, V)) return 0;
    return arrival_layout(B, N, V).total;
}

int ersd_race_verify_arrival_tree_strided(const void* draft_logits, int64_t draft_row_stride,
                                          const void* target_logits, int64_t target_row_stride, ersd_dtype dt,
                                          int32_t B, int32_t N, int32_t V, const int32_t* parent, const int32_t* rank,
                                          float temperature, uint64_t seed, int32_t* draft_tokens,
                                          int32_t* target_tokens, int32_t* accept_len, int32_t* accept_node,
                                          int32_t* emitted, void* workspace, size_t workspace_bytes, void* stream) {
    if (!parent || !rank || !draft_tokens || !target_tokens || !accept_len || !accept_node || !emitted || !workspace)
        return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    if (!arrival_sizes_ok(B, N, V)) return ERSD_ERR_INVALID_ARG;
    const int64_t rows = (int64_t)B * (N + 1);
    if (!stride_ok(draft_row_stride, V, rows) || !stride_ok(target_row_stride, V, rows)) return ERSD_ERR_INVALID_ARG;
    if (workspace_bytes < arrival_layout(B, N, V).total) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    return launch_arrival_tree(draft_logits, draft_row_stride, target_logits, target_row_stride, dt, B, N, V, parent,
                               rank, temperature, seed, draft_tokens, target_tokens, accept_len, accept_node, emitted,
                               workspace, stream);
}

size_t ersd_arrival_tree_plan_bytes(int32_t N) {
    if (N < 1 || N > kMaxArrNodes) return 0;
    return plan_layout(N).total;
}

int ersd_arrival_tree_prepare(const int32_t* parent, const int32_t* rank, int32_t N, void* plan, size_t plan_bytes,
                              void* stream) {
    if (!parent || !rank || !plan) return ERSD_ERR_NULL_POINTER;
    if (N < 1 || N > kMaxArrNodes) return ERSD_ERR_INVALID_ARG;
    if ((uintptr_t)plan & 15) return ERSD_ERR_MISALIGNED;
    const PlanLayout pl = plan_layout(N);
    if (plan_bytes < pl.total) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    char* pb = static_cast<char*>(plan);
    ArrMeta meta{};
    meta.valid = reinterpret_cast<int32_t*>(pb + pl.valid);
    meta.need = reinterpret_cast<int32_t*>(pb + pl.need);
    meta.wprefix = reinterpret_cast<uint32_t*>(pb + pl.wprefix);
    hipLaunchKernelGGL(arrival_meta_kernel, dim3(1), dim3(kThreads), 0, static_cast<hipStream_t>(stream), parent, rank,
                       N, meta);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int ersd_race_verify_arrival_tree_prepared(const void* draft_logits, int64_t draft_row_stride,
                                           const void* target_logits, int64_t target_row_stride, ersd_dtype dt,
                                           int32_t B, int32_t N, int32_t V, const int32_t* parent, const int32_t* rank,
                                           const void* plan, size_t plan_bytes, float temperature, uint64_t seed,
                                           int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                                           int32_t* accept_node, int32_t* emitted, void* workspace,
                                           size_t workspace_bytes, void* stream) {
    if (!parent || !rank || !plan || !draft_tokens || !target_tokens || !accept_len || !accept_node || !emitted ||
        !workspace)
        return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    if ((uintptr_t)plan & 15) return ERSD_ERR_MISALIGNED;
    if (!arrival_sizes_ok(B, N, V)) return ERSD_ERR_INVALID_ARG;
    const int64_t rows = (int64_t)B * (N + 1);
    if (!stride_ok(draft_row_stride, V, rows) || !stride_ok(target_row_stride, V, rows)) return ERSD_ERR_INVALID_ARG;
    if (workspace_bytes < arrival_layout(B, N, V).total || plan_bytes < plan_layout(N).total)
        return ERSD_ERR_WORKSPACE_TOO_SMALL;
    return launch_arrival_tree(draft_logits, draft_row_stride, target_logits, target_row_stride, dt, B, N, V, parent,
                               rank, temperature, seed, draft_tokens, target_tokens, accept_len, accept_node, emitted,
                               workspace, stream, plan);
}

int ersd_race_verify_arrival_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B,
                                  int32_t N, int32_t V, const int32_t* parent, const int32_t* rank, float temperature,
                                  uint64_t seed, int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                                  int32_t* accept_node, int32_t* emitted, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    return ersd_race_verify_arrival_tree_strided(draft_logits, V, target_logits, V, dt, B, N, V, parent, rank,
                                                 temperature, seed, draft_tokens, target_tokens, accept_len,
                                                 accept_node, emitted, workspace, workspace_bytes, stream);
}

int ersd_arrival_tree_validate_host(const int32_t* parent_host, const int32_t* rank_host, int32_t N) {
    if (!parent_host || !rank_host || N < 1 || N > kMaxArrNodes) return 0;
    for (int32_t n = 0; n < N; ++n) {
        if (parent_host[n] < -1 || parent_host[n] >= n || rank_host[n] < 0 || rank_host[n] >= kMaxRank) return 0;
        for (int32_t o = 0; o < n; ++o)
            if (parent_host[o] == parent_host[n] && rank_host[o] == rank_host[n]) return 0;
    }
    return 1;
}

int ersd_max_rank(void) { return kMaxRank; }

size_t ersd_race_workspace_bytes(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, ersd_dtype dt) {
    if (dt != ERSD_F32 && dt != ERSD_BF16) return 0;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return 0;
    return workspace_for(g);
}

int ersd_race_stage_races(int variant, const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B,
                          int32_t m, int32_t k_or_N, int32_t V, float temperature, uint64_t seed, void* workspace,
                          size_t workspace_bytes, void* stream) {
    if (!workspace) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return ERSD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_for(g)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    return launch_races(draft_logits, target_logits, dt, g, temperature, seed, workspace, workspace_bytes, stream);
}

int ersd_race_stage_accept(int variant, ersd_dtype dt, int32_t B, int32_t m, int32_t k_or_N, int32_t V,
                           float temperature, const int32_t* parent, int32_t* draft_tokens, int32_t* target_tokens, int32_t* accept_len,
                           int32_t* best_draft, int32_t* best_len, int32_t* accept_node, const void* workspace,
                           size_t workspace_bytes, void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len || !workspace) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_TREE && !parent) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_MULTI && (!best_draft || !best_len)) return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (!(temperature > 0.0f) || !std::isfinite(temperature)) return ERSD_ERR_INVALID_ARG;
    if ((uintptr_t)workspace & 15) return ERSD_ERR_MISALIGNED;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return ERSD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_for(g)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    if (variant != ERSD_VARIANT_MULTI) { best_draft = nullptr; best_len = nullptr; }
    if (variant != ERSD_VARIANT_TREE) { parent = nullptr; accept_node = nullptr; }
    return launch_finish(variant, g, dt, temperature, parent, draft_tokens, target_tokens, accept_len, best_draft,
                         best_len, accept_node, workspace, workspace_bytes, stream);
}

// The three fused calls share one body: sizes and strides checked on the host, then race and finishing kernels.
static int verify_any(int variant, const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                      int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t m, int32_t k_or_N, int32_t V,
                      const int32_t* parent, float temperature, uint64_t seed, int32_t* draft_tokens,
                      int32_t* target_tokens, int32_t* accept_len, int32_t* best_draft, int32_t* best_len,
                      int32_t* accept_node, void* workspace, size_t workspace_bytes, void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len || !workspace) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_MULTI && (!best_draft || !best_len)) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_TREE && !parent) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, V, g)) return ERSD_ERR_INVALID_ARG;
    if (!stride_ok(draft_row_stride, V, (int64_t)g.B * g.m * g.kd) ||
        !stride_ok(target_row_stride, V, (int64_t)g.B * g.m * g.kt))
        return ERSD_ERR_INVALID_ARG;
    g.qstride = draft_row_stride;
    g.pstride = target_row_stride;
    if (workspace_bytes < workspace_for(g)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    return launch(draft_logits, target_logits, dt, g, temperature, seed, variant, parent, draft_tokens, target_tokens,
                  accept_len, best_draft, best_len, accept_node, workspace, workspace_bytes, stream);
}

int ersd_race_verify_strided(const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                             int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t k, int32_t V,
                             float temperature, uint64_t seed, int32_t* draft_tokens, int32_t* target_tokens,
                             int32_t* accept_len, void* workspace, size_t workspace_bytes, void* stream) {
    return verify_any(ERSD_VARIANT_SEQUENCE, draft_logits, draft_row_stride, target_logits, target_row_stride, dt, B, 1,
                      k, V, nullptr, temperature, seed, draft_tokens, target_tokens, accept_len, nullptr, nullptr,
                      nullptr, workspace, workspace_bytes, stream);
}

int ersd_race_verify_multi_strided(const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                                   int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t m, int32_t k,
                                   int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens,
                                   int32_t* target_tokens, int32_t* accept_len, int32_t* best_draft,
                                   int32_t* best_len, void* workspace, size_t workspace_bytes, void* stream) {
    return verify_any(ERSD_VARIANT_MULTI, draft_logits, draft_row_stride, target_logits, target_row_stride, dt, B, m, k,
                      V, nullptr, temperature, seed, draft_tokens, target_tokens, accept_len, best_draft, best_len,
                      nullptr, workspace, workspace_bytes, stream);
}

int ersd_race_verify_tree_strided(const void* draft_logits, int64_t draft_row_stride, const void* target_logits,
                                  int64_t target_row_stride, ersd_dtype dt, int32_t B, int32_t N, int32_t V,
                                  const int32_t* parent, float temperature, uint64_t seed, int32_t* draft_tokens,
                                  int32_t* target_tokens, int32_t* accept_len, int32_t* accept_node, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    return verify_any(ERSD_VARIANT_TREE, draft_logits, draft_row_stride, target_logits, target_row_stride, dt, B, 1, N,
                      V, parent, temperature, seed, draft_tokens, target_tokens, accept_len, nullptr, nullptr,
                      accept_node, workspace, workspace_bytes, stream);
}

int ersd_noalloc_prepare(void) {
    void* ptr = nullptr;
    const int rc = scratch_of_current_device(&ptr);
    if (rc != ERSD_OK) return rc;
    if (race_blocks(ERSD_F32) < 1 || race_blocks(ERSD_BF16) < 1) return ERSD_ERR_HIP;  // the occupancy queries, cached
    return ERSD_OK;
}

int ersd_race_verify_noalloc(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t k,
                             int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens,
                             int32_t* target_tokens, int32_t* accept_len, void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(draft_logits, target_logits, dt, temperature, nullptr);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    if (!geometry(ERSD_VARIANT_SEQUENCE, B, 1, k, V, g)) return ERSD_ERR_INVALID_ARG;
    if (workspace_for(g) > kScratchBytes) return ERSD_ERR_SCRATCH_TOO_SMALL;
    void* ptr = nullptr;  // the device address of the library's scratch array on the current device
    const int rs = scratch_of_current_device(&ptr);
    if (rs != ERSD_OK) return rs;
    return launch(draft_logits, target_logits, dt, g, temperature, seed, ERSD_VARIANT_SEQUENCE, nullptr, draft_tokens,
                  target_tokens, accept_len, nullptr, nullptr, nullptr, ptr, kScratchBytes, stream);
}

int ersd_race_verify(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t k,
                     int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens, int32_t* target_tokens,
                     int32_t* accept_len, void* workspace, size_t workspace_bytes, void* stream) {
    return ersd_race_verify_strided(draft_logits, V, target_logits, V, dt, B, k, V, temperature, seed, draft_tokens,
                                    target_tokens, accept_len, workspace, workspace_bytes, stream);
}

int ersd_race_verify_multi(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t m,
                           int32_t k, int32_t V, float temperature, uint64_t seed, int32_t* draft_tokens,
                           int32_t* target_tokens, int32_t* accept_len, int32_t* best_draft, int32_t* best_len,
                           void* workspace, size_t workspace_bytes, void* stream) {
    return ersd_race_verify_multi_strided(draft_logits, V, target_logits, V, dt, B, m, k, V, temperature, seed,
                                          draft_tokens, target_tokens, accept_len, best_draft, best_len, workspace,
                                          workspace_bytes, stream);
}

int ersd_race_verify_tree(const void* draft_logits, const void* target_logits, ersd_dtype dt, int32_t B, int32_t N,
                          int32_t V, const int32_t* parent, float temperature, uint64_t seed, int32_t* draft_tokens,
                          int32_t* target_tokens, int32_t* accept_len, int32_t* accept_node, void* workspace,
                          size_t workspace_bytes, void* stream) {
    return ersd_race_verify_tree_strided(draft_logits, V, target_logits, V, dt, B, N, V, parent, temperature, seed,
                                         draft_tokens, target_tokens, accept_len, accept_node, workspace,
                                         workspace_bytes, stream);
}

int ersd_race_sample_strided(const void* logits, int64_t row_stride, ersd_dtype dt, int32_t B, int32_t m,
                             int32_t npos, int32_t V, int32_t pos0, float temperature, uint64_t seed, int32_t* tokens,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!tokens || !workspace) return ERSD_ERR_NULL_POINTER;
    const int rc = check_common(logits, logits, dt, temperature, workspace);
    if (rc != ERSD_OK) return rc;
    Geometry g;
    g.B = B; g.m = m; g.kd = 0; g.kt = npos; g.V = V;  // every row is raced on its own
    g.qstride = g.pstride = row_stride;
    if (npos < 1 || pos0 < 0 || (int64_t)pos0 + npos > 0x7fffffff || !sizes_ok(B, m, 1, npos, V) ||
        !stride_ok(row_stride, V, (int64_t)B * m * npos))
        return ERSD_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_for(g)) return ERSD_ERR_WORKSPACE_TOO_SMALL;
    const int rr = launch_races(nullptr, logits, dt, g, temperature, seed, workspace, workspace_bytes, stream,
                                (uint32_t)pos0);
    if (rr != ERSD_OK) return rr;
    return launch_finish(-1, g, dt, temperature, nullptr, nullptr, tokens, nullptr, nullptr, nullptr, nullptr,
                         workspace, workspace_bytes, stream);
}

int ersd_race_sample(const void* logits, ersd_dtype dt, int32_t B, int32_t m, int32_t npos, int32_t V, int32_t pos0,
                     float temperature, uint64_t seed, int32_t* tokens, void* workspace, size_t workspace_bytes,
                     void* stream) {
    return ersd_race_sample_strided(logits, V, dt, B, m, npos, V, pos0, temperature, seed, tokens, workspace,
                                    workspace_bytes, stream);
}

size_t ersd_race_sample_workspace_bytes(int32_t B, int32_t m, int32_t npos, int32_t V, ersd_dtype dt) {
    if (dt != ERSD_F32 && dt != ERSD_BF16) return 0;
    if (npos < 1 || !sizes_ok(B, m, 1, npos, V)) return 0;
    Geometry g;
    g.B = B; g.m = m; g.kd = 0; g.kt = npos; g.V = V;
    g.qstride = g.pstride = 0;
    return workspace_for(g);
}

int ersd_accept_lengths(int variant, int32_t B, int32_t m, int32_t k_or_N, const int32_t* parent,
                        const int32_t* draft_tokens, const int32_t* target_tokens, int32_t* accept_len,
                        int32_t* best_draft, int32_t* best_len, int32_t* accept_node, void* stream) {
    if (!draft_tokens || !target_tokens || !accept_len) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_TREE && !parent) return ERSD_ERR_NULL_POINTER;
    if (variant == ERSD_VARIANT_MULTI && (!best_draft || !best_len)) return ERSD_ERR_NULL_POINTER;
    Geometry g;
    if (!geometry(variant, B, m, k_or_N, 8, g)) return ERSD_ERR_INVALID_ARG;  // the vocabulary size plays no role
    FinishArgs f{};
    f.part = make_part(g, 1, 0, 0);
    f.out = nullptr;
    f.T = 1.0;
    f.m = g.m;
    f.variant = variant;
    f.parent = variant == ERSD_VARIANT_TREE ? parent : nullptr;
    f.draft_tokens = const_cast<int32_t*>(draft_tokens);   // read only by accept_kernel
    f.target_tokens = const_cast<int32_t*>(target_tokens);
    f.accept_len = accept_len;
    f.best_draft = variant == ERSD_VARIANT_MULTI ? best_draft : nullptr;
    f.best_len = variant == ERSD_VARIANT_MULTI ? best_len : nullptr;
    f.accept_node = variant == ERSD_VARIANT_TREE ? accept_node : nullptr;
    hipLaunchKernelGGL(accept_kernel, dim3((uint32_t)g.B), dim3(kThreads), 0, static_cast<hipStream_t>(stream), f);
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
}

int ersd_read_probe(const void* a, size_t a_bytes, const void* b, size_t b_bytes, void* sink, void* stream) {
    if (!a || !sink || (b_bytes && !b)) return ERSD_ERR_NULL_POINTER;
    if (((uintptr_t)a & 15) || ((uintptr_t)b & 15) || ((uintptr_t)sink & 3)) return ERSD_ERR_MISALIGNED;
    if ((a_bytes & 15) || (b_bytes & 15) || a_bytes == 0) return ERSD_ERR_INVALID_ARG;
    const int blocks = race_blocks(ERSD_BF16);
    if (blocks < 1) return ERSD_ERR_HIP;
    hipLaunchKernelGGL(read_probe_kernel, dim3((uint32_t)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(a), (uint64_t)(a_bytes / 16), static_cast<const u32x4*>(b),
                       (uint64_t)(b_bytes / 16), static_cast<uint32_t*>(sink));
    return hipGetLastError() == hipSuccess ? ERSD_OK : ERSD_ERR_HIP;
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

int ersd_plan_describe_host(int variant, int32_t B, int32_t m, int32_t k_or_N, int32_t V, ersd_dtype dt,
                            uint32_t blocks, uint32_t* out_G, uint32_t* out_nslot, uint32_t* out_seg_cost,
                            uint64_t* block_start, uint32_t* row_first, uint32_t* row_last) {
    Geometry g;
    if (!out_G || !out_nslot) return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (blocks < 1 || blocks > kMaxBlocks || !geometry(variant, B, m, k_or_N, V, g)) return ERSD_ERR_INVALID_ARG;
    const Part p = make_part(g, blocks, seg_cost_for(dt), align_mask_for(dt));
    *out_G = p.G;
    *out_nslot = p.nslot;
    if (out_seg_cost) *out_seg_cost = p.S;
    if (block_start)
        for (uint32_t b = 0; b <= p.G; ++b) {
            const PartPos s = part_start_pos(p, b);
            block_start[b] = s.row * p.V8 + s.grp;
        }
    if (row_first && row_last)
        for (uint64_t r = 0; r < p.rows; ++r) {
            row_first[r] = part_first_block(p, r / p.kt, (uint32_t)(r % p.kt));
            row_last[r] = part_last_block(p, r / p.kt, (uint32_t)(r % p.kt));
        }
    return ERSD_OK;
}

int ersd_arrival_plan_describe_host(int32_t B, int32_t N, int32_t V, ersd_dtype dt, const int32_t* need_host,
                                    uint32_t blocks, uint32_t* out_G, uint32_t* out_nslot, uint64_t* block_start,
                                    uint32_t* row_first, uint32_t* row_last) {
    if (!need_host || !out_G || !out_nslot) return ERSD_ERR_NULL_POINTER;
    if (dt != ERSD_F32 && dt != ERSD_BF16) return ERSD_ERR_UNSUPPORTED_DTYPE;
    if (blocks < 1 || blocks > kMaxBlocks || !arrival_sizes_ok(B, N, V)) return ERSD_ERR_INVALID_ARG;
    const int32_t C = N + 1;
    // the weight table as the tree-shape kernel writes it: a context with a draft row costs as a pair row
    uint32_t* wprefix = new (std::nothrow) uint32_t[(size_t)C + 1];
    if (!wprefix) return ERSD_ERR_INVALID_ARG;
    wprefix[0] = 0;
    for (int32_t c = 0; c < C; ++c) wprefix[c + 1] = wprefix[c] + (need_host[c] > 0 ? kWPair : kWSingle);
    Part p = make_arrival_part(B, C, V, blocks, wprefix, dt);
    p.Us = (uint64_t)wprefix[C] * p.V8;   // what part_on_device reads from the table
    p.U = p.Us * (uint64_t)B;
    *out_G = p.G;
    *out_nslot = p.nslot;
    if (block_start)
        for (uint32_t b = 0; b <= p.G; ++b) {
            const PartPos s = part_start_pos(p, b);
            block_start[b] = s.row * p.V8 + s.grp;
        }
    if (row_first && row_last)
        for (uint64_t r = 0; r < p.rows; ++r) {
            row_first[r] = part_first_block(p, r / p.kt, (uint32_t)(r % p.kt));
            row_last[r] = part_last_block(p, r / p.kt, (uint32_t)(r % p.kt));
        }
    delete[] wprefix;
    return ERSD_OK;
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
        case ERSD_ERR_SCRATCH_TOO_SMALL: return "job needs more scratch memory than the allocation-free entry point holds";
        default: return "unknown status";
    }
}

int ersd_philox_rounds(void) { return kPhiloxRounds; }

void ersd_test_hooks_set(const ersd_test_hooks* h) {
    g_hook_blocks.store(h ? h->force_blocks : 0);
    g_hook_exhaustive.store(h ? h->exhaustive : 0);
    g_hook_seg_cost.store(h ? h->seg_cost_units : -1);
    g_hook_align.store(h ? h->align_groups : -1);
}

int ersd_version(void) { return 410; }

}  // extern "C"
