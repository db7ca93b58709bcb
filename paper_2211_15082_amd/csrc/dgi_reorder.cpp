// Host side of node reordering (Section 4.2 of the DGI paper): produce perm_new_of_old so that nodes with
// consecutive new ids, which form a batch, tend to share in-neighbours.  Any bijection is a correct
// answer for inference; the choices below only affect locality.
//
//  DEGREE : descending in-degree, ties by old id (the "Degree Sorting" comparison point of Section 5.3).
//  BFS_RCM: Cuthill-McKee enumeration on the undirected structure (u ~ v if either direction is stored),
//           reversed at the end (the paper's RCMK).  The paper leaves the details open; here every
//           connected component starts at an unvisited node of minimum undirected degree, and the
//           unvisited neighbours of a dequeued node are appended in ascending (degree, old id) order.  After
//           kMaxBfsComponents components the remaining nodes are appended in (degree, id) order.
//  RANDOM : seeded Fisher-Yates shuffle.
//  COMMUNITY: synchronous label propagation on the undirected structure, then ids by (label, old id).  The rule, which
//           the device kernels follow to the letter: labels start as the node ids; in round r the nodes whose id has
//           the parity of r take a new label, the others keep theirs (two half-steps never flip-flop); a node's
//           neighbour list is its in-neighbours in stored order followed by its out-neighbours in ascending id, with
//           multiplicity; the list is read in chunks of 64, a chunk's winner is its most frequent label (ties: the
//           smallest label), and chunk winners are merged in order: the same label as the running winner adds its
//           count, a different one replaces it only with a strictly larger count.
#include <algorithm>
#include <numeric>
#include <vector>

#include "dgi_internal.h"

namespace dgi {
namespace {

inline uint64_t splitmix64(uint64_t& s) {
    uint64_t z = (s += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

void degree_order(int64_t N, const int64_t* indptr, int32_t* perm) {
    std::vector<int32_t> order((size_t)N);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return indptr[a + 1] - indptr[a] > indptr[b + 1] - indptr[b];
    });
    for (int64_t r = 0; r < N; ++r) perm[order[r]] = (int32_t)r;
}

void random_order(int64_t N, uint64_t seed, int32_t* perm) {
    std::iota(perm, perm + N, 0);
    uint64_t s = seed ^ 0x5851f42d4c957f2dull;
    for (int64_t i = N - 1; i > 0; --i) {
        const int64_t j = (int64_t)(splitmix64(s) % (uint64_t)(i + 1));
        std::swap(perm[i], perm[j]);
    }
}

void rcm_order(int64_t N, const int64_t* indptr, const int32_t* indices, int32_t* perm) {
    // undirected adjacency with multiplicity: every stored edge u->v contributes v to adj[u] and u to adj[v]
    std::vector<int64_t> off((size_t)N + 1, 0);
    for (int64_t v = 0; v < N; ++v) {
        off[v + 1] += indptr[v + 1] - indptr[v];
        for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) off[(int64_t)indices[e] + 1] += 1;
    }
    for (int64_t v = 0; v < N; ++v) off[v + 1] += off[v];
    std::vector<int32_t> adj((size_t)off[N]);
    {
        std::vector<int64_t> cur(off.begin(), off.end() - 1);
        for (int64_t v = 0; v < N; ++v)
            for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) {
                const int32_t u = indices[e];
                adj[cur[v]++] = u;
                adj[cur[u]++] = (int32_t)v;
            }
    }
    auto deg = [&](int32_t x) { return off[(int64_t)x + 1] - off[x]; };
    std::vector<int32_t> by_degree((size_t)N);
    std::iota(by_degree.begin(), by_degree.end(), 0);
    std::stable_sort(by_degree.begin(), by_degree.end(), [&](int32_t a, int32_t b) { return deg(a) < deg(b); });
    std::vector<char> seen((size_t)N, 0);
    std::vector<int32_t> order;
    order.reserve((size_t)N);
    std::vector<int32_t> fresh;
    int components = 0;
    for (int64_t s = 0; s < N; ++s) {
        const int32_t start = by_degree[s];
        if (seen[start]) continue;
        if (components++ >= kMaxBfsComponents) {  // leftovers: (degree, id) order, no more searches
            seen[start] = 1;
            order.push_back(start);
            continue;
        }
        seen[start] = 1;
        size_t head = order.size();
        order.push_back(start);
        while (head < order.size()) {
            const int32_t x = order[head++];
            fresh.clear();
            for (int64_t e = off[x]; e < off[(int64_t)x + 1]; ++e) {
                const int32_t y = adj[e];
                if (!seen[y]) { seen[y] = 1; fresh.push_back(y); }
            }
            std::sort(fresh.begin(), fresh.end(), [&](int32_t a, int32_t b) {
                const int64_t da = deg(a), db = deg(b);
                return da != db ? da < db : a < b;
            });
            order.insert(order.end(), fresh.begin(), fresh.end());
        }
    }
    for (int64_t r = 0; r < N; ++r) perm[order[r]] = (int32_t)(N - 1 - r);  // reversed enumeration
}

void community_order(int64_t N, const int64_t* indptr, const int32_t* indices, int32_t* perm) {
    // out-neighbour lists in ascending destination id (edges are visited by ascending destination row)
    std::vector<int64_t> optr((size_t)N + 1, 0);
    for (int64_t e = 0; e < indptr[N]; ++e) optr[(int64_t)indices[e] + 1] += 1;
    for (int64_t v = 0; v < N; ++v) optr[v + 1] += optr[v];
    std::vector<int32_t> oidx((size_t)indptr[N]);
    {
        std::vector<int64_t> cur(optr.begin(), optr.end() - 1);
        for (int64_t v = 0; v < N; ++v)
            for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) oidx[cur[indices[e]]++] = (int32_t)v;
    }
    std::vector<int32_t> lab((size_t)N), nxt((size_t)N), chunk;
    std::iota(lab.begin(), lab.end(), 0);
    for (int r = 0; r < DGI_COMMUNITY_ROUNDS; ++r) {
        for (int64_t v = 0; v < N; ++v) {
            nxt[v] = lab[v];
            if (((v ^ r) & 1) != 0) continue;
            const int64_t din = indptr[v + 1] - indptr[v], total = din + (optr[v + 1] - optr[v]);
            int32_t best = -1;
            int64_t cnt = 0;
            for (int64_t base = 0; base < total; base += 64) {
                chunk.clear();
                for (int64_t j = base; j < std::min(total, base + 64); ++j)
                    chunk.push_back(lab[j < din ? indices[indptr[v] + j] : oidx[optr[v] + (j - din)]]);
                int32_t w = -1;
                int64_t c = 0;
                for (int32_t a : chunk) {
                    const int64_t ca = std::count(chunk.begin(), chunk.end(), a);
                    if (ca > c || (ca == c && a < w)) { w = a; c = ca; }
                }
                if (w == best) cnt += c;
                else if (c > cnt) { best = w; cnt = c; }
            }
            if (total > 0) nxt[v] = best;
        }
        lab.swap(nxt);
    }
    std::vector<int32_t> order((size_t)N);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return lab[a] < lab[b]; });
    for (int64_t r = 0; r < N; ++r) perm[order[r]] = (int32_t)r;
}

}  // namespace

dgi_status_t reorder_permutation(int64_t N, const int64_t* indptr, const int32_t* indices, int method, uint64_t seed,
                                 int32_t* perm) {
    DGI_REQUIRE(N >= 0 && indptr && perm, DGI_ERR_INVALID_ARG, "reorder: bad argument");
    if (N == 0) return DGI_OK;
    switch (method) {
        case DGI_REORDER_NONE: std::iota(perm, perm + N, 0); return DGI_OK;
        case DGI_REORDER_DEGREE: degree_order(N, indptr, perm); return DGI_OK;
        case DGI_REORDER_RANDOM: random_order(N, seed, perm); return DGI_OK;
        case DGI_REORDER_BFS_RCM:
            DGI_REQUIRE(indices || indptr[N] == 0, DGI_ERR_INVALID_ARG, "reorder: indices is NULL");
            rcm_order(N, indptr, indices, perm);
            return DGI_OK;
        case DGI_REORDER_COMMUNITY:
            DGI_REQUIRE(indices || indptr[N] == 0, DGI_ERR_INVALID_ARG, "reorder: indices is NULL");
            community_order(N, indptr, indices, perm);
            return DGI_OK;
    }
    set_error("reorder: unknown method %d", method);
    return DGI_ERR_INVALID_ARG;
}

}  // namespace dgi
