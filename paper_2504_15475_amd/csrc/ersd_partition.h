// How the rows of one call are shared out: all rows are laid end to end in 8-token groups, weighted by what a group
// costs, with a fixed charge in front of every row (a workgroup that starts a second row pays for an empty load
// pipeline, a new bound and a hand-over: several microseconds), and cut into G equal shares, one per workgroup.
// Host and device evaluate the same functions, so the race kernel (which part is mine, which slot do I write),
// the finishing kernels (which slots does a row have) and the host (workspace size, ersd_plan_describe_host)
// agree by construction.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ersd_part {

#ifndef ERSD_W_PAIR
#define ERSD_W_PAIR 10
#define ERSD_W_SINGLE 5
#endif
// Relative cost of one group in a pair row / target-only row: what it costs to read them.  (While the filter was
// bound by its arithmetic a target-only group, with a generator word per logit, cost 0.7 of a pair group; now a
// share made of target-only rows alone runs in 0.45 to 0.5 of the time of a share of pair rows with as many groups.)
constexpr uint32_t kWPair = ERSD_W_PAIR, kWSingle = ERSD_W_SINGLE;
constexpr uint64_t kMinQuota = 64 * kWPair * 16;     // cost units a workgroup gets at least (16 pair iterations of a wave)

// Balanced partition of the concatenated rows (in 8-token groups) over G workgroups.  Shared by the race
// kernel (which part is mine, which slot do I write) and the finishing kernel (which slots does a row have).
struct Part {
    uint64_t U;           // total cost units
    uint64_t Us;          // cost units per sequence
    uint64_t pair_units;  // cost units of the pair rows of one sequence
    uint32_t S;           // cost units charged to every row start (0 with a weight table)
    uint32_t amask;       // shares start at groups that are multiples of amask + 1 (a power of two): whole cache lines
    uint32_t Lp, Ls;      // cost units of a whole pair row / target-only row: S + weight * V8
    uint64_t rows;        // target rows = races
    uint32_t V8;          // groups per row
    uint32_t kd, kt;      // draft rows / target rows per sequence
    uint32_t G;           // workgroups
    uint32_t nslot;       // partial slots per (row, side)
    // Every workgroup works out its share before its first load, and integer division is a long instruction
    // sequence on this hardware.  When all cost units fit in 32 bits (fast != 0) the quotients below are taken by
    // multiplication with reciprocals prepared on the host (see magic_of); otherwise by plain 64-bit division.
    uint32_t fast;
    uint32_t q, r;        // U / G and U % G: share b starts at unit b * q + (b * r) / G = floor(b * U / G)
    uint64_t m_G, m_q, m_Us, m_pair_row, m_single_row, m_kt;  // reciprocals of G, q, Us, Lp, Ls, kt
    // Arrival trees: which contexts have a draft row is known on the device only.  wprefix[c] = summed weights of
    // the contexts before c (kt + 1 entries, device memory); nullptr for the closed-form layouts above.
    const uint32_t* wprefix;
};

// Division of a 32-bit number by a fixed 32-bit divisor d through its 64-bit reciprocal m = floor(2^64 / d) + 1:
// floor(n / d) = floor(n * m / 2^64) for every n < 2^32 (the product overshoots n / d by less than 2^-32, which
// cannot reach the next integer because the fraction of n / d is at most 1 - 1/d).  m == 0 stands for d == 1.
inline uint64_t magic_of(uint64_t d) { return d <= 1 ? 0 : ~(uint64_t)0 / d + 1; }
__host__ __device__ inline uint32_t magic_div(uint32_t n, uint64_t m) {
    if (!m) return n;
    const uint64_t lo = (uint64_t)n * (uint32_t)m, hi = (uint64_t)n * (uint32_t)(m >> 32);
    return (uint32_t)((hi + (lo >> 32)) >> 32);
}

// context whose cost units contain weighted position wpos (in units of one group): largest c with wprefix[c] <= wpos
__host__ __device__ inline uint32_t part_table_row(const Part& p, uint64_t wpos) {
    uint32_t lo = 0, hi = p.kt;  // answer in [lo, hi)
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if ((uint64_t)p.wprefix[mid] <= wpos) lo = mid;
        else hi = mid;
    }
    return lo;
}

struct PartPos {
    uint64_t row;   // global row = seq * kt + j
    uint64_t seq;
    uint32_t j;     // row within the sequence
    uint32_t grp;   // group within the row
};

// group that contains cost unit u (u >= U: the end)
__host__ __device__ inline PartPos part_unit_to_pos(const Part& p, uint64_t u) {
    PartPos o;
    if (u >= p.U) {
        o.row = p.rows;
        o.seq = p.fast ? magic_div((uint32_t)p.rows, p.m_kt) : p.rows / p.kt;
        o.j = 0;
        o.grp = 0;
        return o;
    }
    if (p.fast) {  // closed-form layout, everything below 2^32
        const uint32_t u32 = (uint32_t)u, seq = magic_div(u32, p.m_Us), rem = u32 - seq * (uint32_t)p.Us;
        o.seq = seq;
        // (a unit inside a row's start charge stands for the row's first group)
        if (rem < (uint32_t)p.pair_units) {
            o.j = magic_div(rem, p.m_pair_row);
            const uint32_t off = rem - o.j * p.Lp;
            o.grp = off < p.S ? 0 : (off - p.S) / kWPair;
        } else {
            const uint32_t r2 = rem - (uint32_t)p.pair_units, jj = magic_div(r2, p.m_single_row);
            o.j = p.kd + jj;
            const uint32_t off = r2 - jj * p.Ls;
            o.grp = off < p.S ? 0 : (off - p.S) / kWSingle;
        }
        o.grp &= ~p.amask;
        o.row = (uint64_t)seq * p.kt + o.j;
        return o;
    }
    const uint64_t seq = u / p.Us, rem = u % p.Us;
    uint64_t row, grp;
    if (p.wprefix) {
        row = part_table_row(p, rem / p.V8);
        grp = (rem - (uint64_t)p.wprefix[row] * p.V8) / (p.wprefix[row + 1] - p.wprefix[row]);
    } else if (rem < p.pair_units) {
        row = rem / p.Lp;
        const uint64_t off = rem % p.Lp;
        grp = off < p.S ? 0 : (off - p.S) / kWPair;
    } else {
        const uint64_t r2 = rem - p.pair_units, off = r2 % p.Ls;
        row = p.kd + r2 / p.Ls;
        grp = off < p.S ? 0 : (off - p.S) / kWSingle;
    }
    o.seq = seq;
    o.j = (uint32_t)row;
    o.grp = (uint32_t)grp & ~p.amask;
    o.row = seq * p.kt + row;
    return o;
}
// first cost unit of workgroup b's share, floor(b * U / G); b == G gives U
__host__ __device__ inline uint64_t part_block_start_unit(const Part& p, uint32_t b) {
    if (p.fast) return (uint64_t)(b * p.q + magic_div(b * p.r, p.m_G));  // b * r < G^2 <= 2^24; the sum is <= U
    return (uint64_t)b * p.U / p.G;
}
// first group of workgroup b's share; b == G gives the end
__host__ __device__ inline PartPos part_start_pos(const Part& p, uint32_t b) {
    return part_unit_to_pos(p, part_block_start_unit(p, b));
}
// first cost unit of the groups of row (seq, j), after the row's start charge, and the weight of a group
__host__ __device__ inline uint64_t part_row_unit(const Part& p, uint64_t seq, uint32_t j, uint32_t* w) {
    if (p.wprefix) {
        *w = p.wprefix[j + 1] - p.wprefix[j];
        return seq * p.Us + (uint64_t)p.wprefix[j] * p.V8;
    }
    *w = j < p.kd ? kWPair : kWSingle;
    return seq * p.Us + p.S + (j < p.kd ? (uint64_t)j * p.Lp : p.pair_units + (uint64_t)(j - p.kd) * p.Ls);
}
// workgroup whose share contains cost unit x < U: the largest b with floor(b * U / G) <= x
__host__ __device__ inline uint32_t part_block_of_unit(const Part& p, uint64_t x) {
    if (p.fast) {
        // b * q <= floor(b * U / G) < b * q + G and q > G (the quota), so the answer is floor(x / q) or one less
        const uint32_t b = magic_div((uint32_t)x, p.m_q);
        if (b >= p.G) return p.G - 1;
        return part_block_start_unit(p, b) <= x ? b : b - 1;
    }
    return (uint32_t)(((x + 1) * p.G - 1) / p.U);
}
// workgroup that holds the first group of row (seq, j): a share starts at the aligned run of groups that contains
// its first unit, so a group belongs to the last share that starts at or before the last unit of the group's run
__host__ __device__ inline uint32_t part_first_block(const Part& p, uint64_t seq, uint32_t j) {
    uint32_t w;
    const uint64_t u0 = part_row_unit(p, seq, j, &w);
    const uint32_t run = p.amask + 1 < p.V8 ? p.amask + 1 : p.V8;  // groups of the row's first run
    return part_block_of_unit(p, u0 + (uint64_t)run * w - 1);
}
// workgroup that holds the last group of row (seq, j)
__host__ __device__ inline uint32_t part_last_block(const Part& p, uint64_t seq, uint32_t j) {
    uint32_t w;
    const uint64_t u1 = part_row_unit(p, seq, j, &w) + (uint64_t)w * p.V8;
    return part_block_of_unit(p, u1 - 1);
}
// number of segment slots of a global row
__host__ __device__ inline uint32_t part_row_slots(const Part& p, uint64_t row) {
    uint64_t seq;
    uint32_t j;
    if (p.fast) {
        const uint32_t s32 = magic_div((uint32_t)row, p.m_kt);
        seq = s32;
        j = (uint32_t)row - s32 * p.kt;
    } else {
        seq = row / p.kt;
        j = (uint32_t)(row % p.kt);
    }
    return part_last_block(p, seq, j) - part_first_block(p, seq, j) + 1;
}

}  // namespace ersd_part
