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

}  // namespace

extern "C" int pk_trie_partition(const int32_t* token_ids, const int32_t* kv_lens, int32_t n,
                                 int32_t min_prefix, int32_t* prefix_ids, int32_t* prefix_lens,
                                 int64_t* saved_tokens) {
    if (n < 0 || min_prefix < 1) return fail("pk_trie_partition: n >= 0 and min_prefix >= 1 required");
    if (n > 0 && (!token_ids || !kv_lens || !prefix_ids || !prefix_lens))
        return fail("pk_trie_partition: NULL pointer");
    std::vector<int64_t> start(static_cast<size_t>(n) + 1, 0);
    for (int32_t i = 0; i < n; ++i) {
        if (kv_lens[i] <= 0) return fail("pk_trie_partition: kv_len must be positive");
        start[i + 1] = start[i] + kv_lens[i];
    }
    for (int32_t i = 0; i < n; ++i) { prefix_ids[i] = -1; prefix_lens[i] = 0; }
    if (saved_tokens) *saved_tokens = 0;
    if (n < 2) return PK_OK;

    auto seq = [&](int32_t i) { return token_ids + start[i]; };
    std::vector<int32_t> idx(static_cast<size_t>(n));
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

    std::vector<Interval> iv;
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
        if (stack.empty()) break;                   // k == n: the root itself was closed
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
    // the root (depth 0) is closed by lcp[n] = -1
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
}
