// Layout of a prepared tree shape (ersd_arrival_tree_prepare), shared by the sources that read one:
// valid[N], need[N + 1], wprefix[N + 2], each 16-byte aligned.
#pragma once
#include <cstddef>
#include <cstdint>

namespace ersd_plan {

inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

struct PlanLayout {
    size_t valid, need, wprefix, total;
};
inline PlanLayout plan_layout(int32_t N) {
    PlanLayout l;
    l.valid = 0;
    l.need = align16(l.valid + (size_t)N * sizeof(int32_t));
    l.wprefix = align16(l.need + (size_t)(N + 1) * sizeof(int32_t));
    l.total = align16(l.wprefix + (size_t)(N + 2) * sizeof(uint32_t));
    return l;
}

}  // namespace ersd_plan
