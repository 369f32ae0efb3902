// libersd, host side: drafting-tree generators for the arrival-tree verification call.
//
// Algorithm 3 of the paper grows the tree that maximises the expected number of accepted drafted tokens, the sum
// of the acceptance probabilities R of its vertices: because a vertex is accepted only if its parent is, R falls
// along every path, so the k best vertices form a tree and can be collected greedily from a priority queue that
// holds, for every vertex taken so far, its first child and its next sibling.  Here R is the 0-th order
// approximation the paper's experiments use (Section 5): R(j_1 .. j_l) = r[j_1] * ... * r[j_l], where r[j] is the
// measured probability that the child holding arrival j is accepted given that its parent was (non-increasing in j).
// Equal values are taken by depth, then by index tuple, so that the result is a function of r and k alone: the k
// vertices with the largest R in the order (R descending, depth, index tuple).

#include <algorithm>
#include <cstdint>
#include <queue>
#include <vector>

#include "ersd.h"

namespace {

struct Entry {
    double value;     // R of the vertex
    int32_t depth;    // number of tokens on its path
    int32_t parent;   // node index of the parent (-1: the root)
    int32_t rank;
};

// Order of the queue.  The parents of queued vertices are nodes of the tree already, so a vertex's index tuple is
// its rank after its parent's tuple, read off the (parent, rank) arrays.
struct Later {
    const int32_t* parent;
    const int32_t* rank;

    void path(const Entry& e, std::vector<int32_t>& out) const {  // index tuple, root first
        out.clear();
        out.push_back(e.rank);
        for (int32_t n = e.parent; n >= 0; n = parent[n]) out.push_back(rank[n]);
        std::reverse(out.begin(), out.end());
    }
    // priority_queue keeps the LARGEST element on top: a is "less" if it must leave later
    bool operator()(const Entry& a, const Entry& b) const {
        if (a.value != b.value) return a.value < b.value;
        if (a.depth != b.depth) return a.depth > b.depth;
        std::vector<int32_t> pa, pb;
        path(a, pa);
        path(b, pb);
        return pa > pb;
    }
};

}  // namespace

extern "C" {

int ersd_tree_build_optimal_host(const double* accept_by_rank, int32_t nr, int32_t k, int32_t* parent, int32_t* rank,
                                 double* node_accept, double* expected_accepted) {
    if (!accept_by_rank || !parent || !rank) return ERSD_ERR_NULL_POINTER;
    if (nr < 1 || k < 1) return ERSD_ERR_INVALID_ARG;
    for (int32_t j = 0; j < nr; ++j) {
        if (!(accept_by_rank[j] >= 0.0 && accept_by_rank[j] <= 1.0)) return ERSD_ERR_INVALID_ARG;
        if (j > 0 && accept_by_rank[j] > accept_by_rank[j - 1]) return ERSD_ERR_INVALID_ARG;
    }
    const Later later{parent, rank};
    std::vector<Entry> store;
    store.reserve((size_t)2 * k + 1);
    std::priority_queue<Entry, std::vector<Entry>, Later> queue(later, std::move(store));
    std::vector<double> value((size_t)k);
    std::vector<int32_t> depth((size_t)k);
    queue.push(Entry{accept_by_rank[0], 1, -1, 0});
    double total = 0.0;
    for (int32_t n = 0; n < k; ++n) {
        const Entry e = queue.top();
        queue.pop();
        parent[n] = e.parent;
        rank[n] = e.rank;
        value[n] = e.value;
        depth[n] = e.depth;
        total += e.value;
        queue.push(Entry{e.value * accept_by_rank[0], e.depth + 1, n, 0});        // first child
        if (e.rank + 1 < nr) {                                                    // next sibling
            const double up = e.parent < 0 ? 1.0 : value[e.parent];
            queue.push(Entry{up * accept_by_rank[e.rank + 1], e.depth, e.parent, e.rank + 1});
        }
    }
    if (node_accept)
        for (int32_t n = 0; n < k; ++n) node_accept[n] = value[n];
    if (expected_accepted) *expected_accepted = total;
    return ERSD_OK;
}

int ersd_tree_build_specinfer_host(int32_t k, int32_t shared, int32_t branches, int32_t* parent, int32_t* rank) {
    if (!parent || !rank) return ERSD_ERR_NULL_POINTER;
    if (k < 1 || shared < 0 || branches < 1) return ERSD_ERR_INVALID_ARG;
    int32_t n = 0;
    for (; n < k && n < shared; ++n) {  // the common prefix: a chain of winners
        parent[n] = n - 1;
        rank[n] = 0;
    }
    std::vector<int32_t> tip((size_t)branches, shared - 1);  // last node of every branch so far
    std::vector<char> started((size_t)branches, 0);
    for (int32_t b = 0; n < k; b = (b + 1) % branches, ++n) {  // the branches grow in turn
        parent[n] = tip[b];
        rank[n] = started[b] ? 0 : b;  // the branches leave the prefix as its arrivals 0, 1, 2, ..; then chains
        started[b] = 1;
        tip[b] = n;
    }
    return ERSD_OK;
}

}  // extern "C"
