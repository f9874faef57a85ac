// Host search for HAGs of a sequential Aggregate (Algorithm 3 with the prefix form of Redundancy).
//
// With ordered neighbour lists only common PREFIXES can be shared (Section 3.1), so the pairs that
// Algorithm 3 may merge are the leading pairs of the current lists.  Merging a pair changes no other
// pair's count: the lists that started with (v1, v2) now start with (w, third element), every other
// list is untouched.  The count of a leading pair is therefore fixed from the moment the pair comes
// into being, and the greedy choice is a plain priority queue over the pairs with count >= 2: no
// recounting, O(|E| log |E|) in all.  A list is never rewritten: it is a head node (an original
// node or the aggregation node standing for the prefix consumed so far) and a position in the
// input's column array.
#include <algorithm>
#include <cstdint>
#include <new>
#include <queue>
#include <string>
#include <tuple>
#include <vector>

#include "hag_internal.hpp"

using namespace hag;

namespace {
struct Group {
    int32_t count, v1, v2;
    int64_t members;   // index into the pool of member lists
};
struct Worse {   // priority queue order: larger count first, then lexicographically smaller (v1, v2)
    bool operator()(const Group &a, const Group &b) const {
        if (a.count != b.count) return a.count < b.count;
        if (a.v1 != b.v1) return a.v1 > b.v1;
        return a.v2 > b.v2;
    }
};
}  // namespace

extern "C" int hag_seq_search(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity, int64_t *n_merges,
                              int32_t *left, int32_t *right, int32_t *redundancy, int64_t *hrowptr, int32_t *hcol) {
    auto fail = [](const char *msg) { set_error(msg); return (int)HAG_EINVAL; };
    if (n < 0 || capacity < 0) return fail("n < 0 or capacity < 0");
    if (!rowptr || !n_merges || !hrowptr) return fail("NULL argument");
    if (rowptr[0] != 0) return fail("rowptr[0] != 0");
    for (int64_t v = 0; v < n; ++v)
        if (rowptr[v + 1] < rowptr[v]) return fail("rowptr is not monotone");
    const int64_t e = rowptr[n];
    if (e > 0 && (!col || !hcol)) return fail("col or hcol is NULL");
    for (int64_t i = 0; i < e; ++i)
        if (col[i] < 0 || col[i] >= n) return fail("col out of range");
    if (capacity > 0 && (!left || !right || !redundancy)) return fail("merge arrays are NULL");
    if (n + std::min(capacity, e) >= (int64_t)INT32_MAX) return fail("n + capacity must be below 2^31");
    try {
        std::vector<int32_t> head(n, -1);
        std::vector<int64_t> pos(n);
        std::vector<std::vector<int32_t>> pool;   // member lists of the groups
        std::priority_queue<Group, std::vector<Group>, Worse> heap;
        // groups of the lists in `who` (all with the same head) by their next element
        auto regroup = [&](std::vector<int32_t> &who, int32_t v1) {
            std::sort(who.begin(), who.end(), [&](int32_t a, int32_t b) {
                const int32_t xa = col[pos[a]], xb = col[pos[b]];
                return xa != xb ? xa < xb : a < b;
            });
            for (size_t i = 0; i < who.size();) {
                size_t j = i;
                while (j < who.size() && col[pos[who[j]]] == col[pos[who[i]]]) ++j;
                if (j - i >= 2) {   // a pair led by a single list can never be merged: its count stays 1
                    pool.emplace_back(who.begin() + i, who.begin() + j);
                    heap.push(Group{(int32_t)(j - i), v1, col[pos[who[i]]], (int64_t)pool.size() - 1});
                }
                i = j;
            }
        };
        {
            std::vector<int32_t> with_pair;
            for (int64_t u = 0; u < n; ++u) {
                if (rowptr[u + 1] > rowptr[u]) head[u] = col[rowptr[u]];
                pos[u] = rowptr[u] + 1;
                if (pos[u] < rowptr[u + 1]) with_pair.push_back((int32_t)u);
            }
            std::sort(with_pair.begin(), with_pair.end(), [&](int32_t a, int32_t b) { return head[a] != head[b] ? head[a] < head[b] : a < b; });
            for (size_t i = 0; i < with_pair.size();) {
                size_t j = i;
                while (j < with_pair.size() && head[with_pair[j]] == head[with_pair[i]]) ++j;
                std::vector<int32_t> same(with_pair.begin() + i, with_pair.begin() + j);
                regroup(same, head[with_pair[i]]);
                i = j;
            }
        }
        int64_t a = 0;
        while (a < capacity && !heap.empty()) {
            const Group g = heap.top();   // count >= 2 by construction: stop when nothing is left
            heap.pop();
            const int32_t w = (int32_t)(n + a);
            left[a] = g.v1;
            right[a] = g.v2;
            redundancy[a] = g.count;
            ++a;
            std::vector<int32_t> who = std::move(pool[(size_t)g.members]);
            std::vector<int32_t> longer;
            for (int32_t u : who) {
                head[u] = w;
                if (++pos[u] < rowptr[u + 1]) longer.push_back(u);
            }
            regroup(longer, w);
        }
        *n_merges = a;
        int64_t out = 0;
        for (int64_t u = 0; u < n; ++u) {
            hrowptr[u] = out;
            if (head[u] >= 0) {
                hcol[out++] = head[u];
                for (int64_t i = pos[u]; i < rowptr[u + 1]; ++i) hcol[out++] = col[i];
            }
        }
        hrowptr[n] = out;
        return HAG_OK;
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return HAG_ENOMEM;
    }
}
