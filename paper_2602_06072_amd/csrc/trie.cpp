// TriePartition from token ids (Alg. 1 Part 2; Sec. 3.2 "Prefix-Aware Grouping and Reuse"): finds
// the shared prefixes P_k of a batch and assigns every request to at most one of them, such that
// the I/O volume of Eq. 5 is smallest: a prefix of d tokens shared by m requests is stored once
// and saves d * (m - 1) tokens.  Host only.
//
// The prefix tree is never built.  The requests are sorted by their token sequences; with the
// longest common prefix of neighbours in that order, every tree node below which at least two
// requests lie is an interval of the sorted order (an "LCP interval"), and the intervals nest like
// the tree.  One pass with a stack enumerates them bottom-up; the best saving of an interval is
// the larger of taking it as one family and the sum over its child intervals.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

#include "plan.h"

namespace {

struct Interval {
    int32_t depth = 0;            // tokens shared by all requests of the interval
    int32_t lo = 0, hi = 0;       // positions in the sorted order
    int64_t best = 0;             // largest saving inside
    bool take = false;            // the interval itself is a family
    std::vector<int32_t> kids;
};

int fail(const char* msg) {
    pk::set_error(msg);
    return PK_EINVAL;
}

// Sorts the requests and enumerates the LCP intervals; iv[0] is the whole batch (depth 0), idx the
// sorted order.  Expects n >= 2 and validated lengths.
void lcp_intervals(const int32_t* token_ids, const int32_t* kv_lens, int32_t n, int32_t min_prefix,
                   std::vector<int32_t>& idx, std::vector<Interval>& iv) {
    std::vector<int64_t> start(static_cast<size_t>(n) + 1, 0);
    for (int32_t i = 0; i < n; ++i) start[i + 1] = start[i] + kv_lens[i];
    auto seq = [&](int32_t i) { return token_ids + start[i]; };
    idx.resize(static_cast<size_t>(n));
    std::iota(idx.begin(), idx.end(), 0);
    std::sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) {
        const int32_t* pa = seq(a); const int32_t* pb = seq(b);
        const int32_t la = kv_lens[a], lb = kv_lens[b], m = std::min(la, lb);
        for (int32_t k = 0; k < m; ++k)
            if (pa[k] != pb[k]) return pa[k] < pb[k];
        if (la != lb) return la < lb;
        return a < b;
    });
    // lcp[k]: common prefix of the requests at sorted positions k-1 and k; lcp[n] ends the scan
    std::vector<int32_t> lcp(static_cast<size_t>(n) + 1, -1);
    for (int32_t k = 1; k < n; ++k) {
        const int32_t a = idx[k - 1], b = idx[k], m = std::min(kv_lens[a], kv_lens[b]);
        const int32_t* pa = seq(a); const int32_t* pb = seq(b);
        int32_t c = 0;
        while (c < m && pa[c] == pb[c]) ++c;
        lcp[k] = c;
    }

    std::vector<int32_t> stack;
    auto close = [&](int32_t v, int32_t hi) {
        Interval& x = iv[static_cast<size_t>(v)];
        x.hi = hi;
        int64_t below = 0;
        for (int32_t c : x.kids) below += iv[static_cast<size_t>(c)].best;
        const int64_t own = x.depth >= min_prefix ? static_cast<int64_t>(x.depth) * (x.hi - x.lo) : 0;
        x.take = own > 0 && own >= below;
        x.best = x.take ? own : below;
    };
    iv.push_back(Interval{});                       // the whole batch, depth 0
    stack.push_back(0);
    for (int32_t k = 1; k <= n; ++k) {
        int32_t lb = k - 1, pending = -1;
        while (!stack.empty() && lcp[k] < iv[static_cast<size_t>(stack.back())].depth) {
            const int32_t v = stack.back();
            stack.pop_back();
            if (pending >= 0) iv[static_cast<size_t>(v)].kids.push_back(pending);
            close(v, k - 1);
            lb = iv[static_cast<size_t>(v)].lo;
            pending = v;
        }
        if (stack.empty()) break;                   // k == n: lcp[n] = -1 closed the root (depth 0) itself
        if (lcp[k] > iv[static_cast<size_t>(stack.back())].depth) {
            Interval x;
            x.depth = lcp[k]; x.lo = lb;
            if (pending >= 0) x.kids.push_back(pending);
            iv.push_back(x);
            stack.push_back(static_cast<int32_t>(iv.size()) - 1);
        } else if (pending >= 0) {
            iv[static_cast<size_t>(stack.back())].kids.push_back(pending);
        }
    }
}

int check_lengths(const char* who, const int32_t* kv_lens, int32_t n) {
    for (int32_t i = 0; i < n; ++i)
        if (kv_lens[i] <= 0) return fail((std::string(who) + ": kv_len must be positive").c_str());
    return PK_OK;
}

}  // namespace

extern "C" int pk_trie_partition(const int32_t* token_ids, const int32_t* kv_lens, int32_t n,
                                 int32_t min_prefix, int32_t* prefix_ids, int32_t* prefix_lens,
                                 int64_t* saved_tokens) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_trie_partition", [&]() -> int {
        if (n < 0 || min_prefix < 1) return fail("pk_trie_partition: n >= 0 and min_prefix >= 1 required");
        if (n > 0 && (!token_ids || !kv_lens || !prefix_ids || !prefix_lens))
            return fail("pk_trie_partition: NULL pointer");
        if (check_lengths("pk_trie_partition", kv_lens, n) != PK_OK) return PK_EINVAL;
        for (int32_t i = 0; i < n; ++i) { prefix_ids[i] = -1; prefix_lens[i] = 0; }
        if (saved_tokens) *saved_tokens = 0;
        if (n < 2) return PK_OK;
        std::vector<int32_t> idx;
        std::vector<Interval> iv;
        lcp_intervals(token_ids, kv_lens, n, min_prefix, idx, iv);
        struct Family { int32_t depth, first; int32_t lo, hi; };
        std::vector<Family> fams;
        std::vector<int32_t> walk{0};
        while (!walk.empty()) {
            const Interval& x = iv[static_cast<size_t>(walk.back())];
            walk.pop_back();
            if (x.take) {
                int32_t first = idx[x.lo];
                for (int32_t p = x.lo; p <= x.hi; ++p) first = std::min(first, idx[p]);
                fams.push_back({x.depth, first, x.lo, x.hi});
            } else {
                for (int32_t c : x.kids) walk.push_back(c);
            }
        }
        std::sort(fams.begin(), fams.end(), [](const Family& a, const Family& b) { return a.first < b.first; });
        int64_t saved = 0;
        for (size_t f = 0; f < fams.size(); ++f) {
            for (int32_t p = fams[f].lo; p <= fams[f].hi; ++p) {
                prefix_ids[idx[p]] = static_cast<int32_t>(f);
                prefix_lens[idx[p]] = fams[f].depth;
            }
            saved += static_cast<int64_t>(fams[f].depth) * (fams[f].hi - fams[f].lo);
        }
        if (saved_tokens) *saved_tokens = saved;
        return PK_OK;
    });
}

// The whole prefix tree as a forest of shared segments: every LCP interval of at least min_prefix
// tokens is a node (Eq. 5 applied at every level: a segment of len tokens above m requests saves
// len * (m - 1)).  Nodes are numbered by (lowest request below, depth), which puts parents first.
extern "C" int pk_trie_tree(const int32_t* token_ids, const int32_t* kv_lens, int32_t n,
                            int32_t min_prefix, int32_t* node_parent, int32_t* node_len,
                            int32_t* n_nodes, int32_t* req_node, int64_t* saved_tokens) {
    return pk::guarded<int>(PK_ENOMEM, PK_EINVAL, "pk_trie_tree", [&]() -> int {
        if (n < 0 || min_prefix < 1) return fail("pk_trie_tree: n >= 0 and min_prefix >= 1 required");
        if (!n_nodes) return fail("pk_trie_tree: n_nodes is NULL");
        if (n > 0 && (!token_ids || !kv_lens || !node_parent || !node_len || !req_node))
            return fail("pk_trie_tree: NULL pointer");
        if (check_lengths("pk_trie_tree", kv_lens, n) != PK_OK) return PK_EINVAL;
        for (int32_t i = 0; i < n; ++i) req_node[i] = -1;
        *n_nodes = 0;
        if (saved_tokens) *saved_tokens = 0;
        if (n < 2) return PK_OK;
        std::vector<int32_t> idx;
        std::vector<Interval> iv;
        lcp_intervals(token_ids, kv_lens, n, min_prefix, idx, iv);

        struct Seg { int32_t first, depth, parent_depth, lo, hi, parent_iv, number; };
        std::vector<Seg> segs;
        std::vector<int32_t> seg_of(iv.size(), -1);
        // top-down: (interval, nearest ancestor that is a node)
        std::vector<std::pair<int32_t, int32_t>> walk{{0, -1}};
        while (!walk.empty()) {
            const int32_t v = walk.back().first;
            int32_t anc = walk.back().second;
            walk.pop_back();
            const Interval& x = iv[static_cast<size_t>(v)];
            if (x.depth >= min_prefix) {
                int32_t first = idx[x.lo];
                for (int32_t p = x.lo; p <= x.hi; ++p) first = std::min(first, idx[p]);
                const int32_t pd = anc >= 0 ? iv[static_cast<size_t>(anc)].depth : 0;
                seg_of[static_cast<size_t>(v)] = static_cast<int32_t>(segs.size());
                segs.push_back({first, x.depth, pd, x.lo, x.hi, anc, 0});
                anc = v;
            }
            for (int32_t c : x.kids) walk.push_back({c, anc});
        }
        std::vector<int32_t> order(segs.size());
        std::iota(order.begin(), order.end(), 0);
        std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            if (segs[a].first != segs[b].first) return segs[a].first < segs[b].first;
            return segs[a].depth < segs[b].depth;
        });
        for (size_t k = 0; k < order.size(); ++k) segs[static_cast<size_t>(order[k])].number = static_cast<int32_t>(k);
        int64_t saved = 0;
        std::vector<int32_t> deepest(static_cast<size_t>(n), 0);
        for (const Seg& sg : segs) {
            node_parent[sg.number] = sg.parent_iv >= 0 ? segs[static_cast<size_t>(seg_of[static_cast<size_t>(sg.parent_iv)])].number : -1;
            node_len[sg.number] = sg.depth - sg.parent_depth;
            saved += static_cast<int64_t>(sg.depth - sg.parent_depth) * (sg.hi - sg.lo);
            for (int32_t p = sg.lo; p <= sg.hi; ++p)
                if (sg.depth > deepest[idx[p]]) { deepest[idx[p]] = sg.depth; req_node[idx[p]] = sg.number; }
        }
        *n_nodes = static_cast<int32_t>(segs.size());
        if (saved_tokens) *saved_tokens = saved;
        return PK_OK;
    });
}
